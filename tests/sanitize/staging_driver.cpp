// Driver for a sanitizer build of the staging-address checker (test infrastructure, CPU only): reads launch shapes
// from stdin ("g M K N cu split_bytes" for a product, "f n Hkv DH causal" for attention), runs the checker on each
// and prints "status loads" per line. Built by the test with g++ -fsanitize=address,undefined together with
// csrc/staging_check.cpp.
#include <cstdio>

extern "C" int dash_check_gemm_staging(int M, int K, int N, int cu, unsigned long long split_bytes, long long* n_loads);
extern "C" int dash_check_flash_staging(int n, int Hkv, int DH, int causal, long long* n_loads);
extern "C" void dash_gemm_launch_plan(int M, int K, int N, int cu, unsigned long long split_bytes, int* out);

int main() {
    char kind;
    while (std::scanf(" %c", &kind) == 1) {
        long long loads = 0;
        int st = -99;
        if (kind == 'g') {
            int M, K, N, cu;
            unsigned long long sb;
            if (std::scanf("%d %d %d %d %llu", &M, &K, &N, &cu, &sb) != 5) return 2;
            st = dash_check_gemm_staging(M, K, N, cu, sb, &loads);
            int plan[10] = {0};
            dash_gemm_launch_plan(M, K, N, cu, sb, plan);
            std::printf("%d %lld %d %d\n", st, loads, plan[0], plan[2]);
        } else if (kind == 'f') {
            int n, Hkv, DH, causal;
            if (std::scanf("%d %d %d %d", &n, &Hkv, &DH, &causal) != 4) return 2;
            st = dash_check_flash_staging(n, Hkv, DH, causal, &loads);
            std::printf("%d %lld\n", st, loads);
        } else {
            return 2;
        }
    }
    return 0;
}
