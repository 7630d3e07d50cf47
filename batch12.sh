R=$GRAFT_REPO_ROOT/_work/exp/run3.sh
N1="f16_t, f32_t, 128, 256, 64, 64, 64, 32, 1, 1, 1, true, 2, false"
N2="f16_t, f32_t, 128, 256, 64, 64, 64, 32, 1, 1, 1, true, 2, true"
K1="f16_t, f32_t, 128, 256, 64, 64, 64, 32, 1, 1, 0, true, 2, true"
A="f16_t, f32_t, 256, 256, 64, 128, 64, 32, 1, 1, 0, true, 2, true"
for c in "$N1" "$N2" "$K1"; do bash $R "$c" 1024 8192 3072 768 4 || exit 1; done
bash $R "$A" 1024 4096 4096 4096 4 || exit 1
