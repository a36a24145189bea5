// Host driver for the CPU emulation build: forward of a whole stack through chebykan_stack_forward.
//   emu_stack_driver <dir> <B> <degree> <n_layers> <w0> <w1> ... <wn>
// <dir> holds x.bin, dy.bin (gradient of the last output) and C0.bin .. C{n-1}.bin; y{l}.bin (layer
// outputs), g{l}.bin (gradient with respect to the input of layer l) and dC{l}.bin are written there.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string>
#include <vector>

#include "../../include/chebykan.h"
#include "../../include/chebykan_tools.h"

static std::vector<float> read_bin(const std::string& path, size_t n)
{
    std::vector<float> v(n);
    FILE* f = fopen(path.c_str(), "rb");
    if (!f || fread(v.data(), sizeof(float), n, f) != n) { fprintf(stderr, "cannot read %s\n", path.c_str()); exit(3); }
    fclose(f);
    return v;
}

int main(int argc, char** argv)
{
    if (argc < 7) { fprintf(stderr, "usage: emu_stack_driver dir B degree n_layers w0 .. wn\n"); return 2; }
    const std::string dir = argv[1];
    const long B = atol(argv[2]);
    const int d = atoi(argv[3]), n = atoi(argv[4]);
    if (argc != 6 + n) { fprintf(stderr, "need n_layers+1 widths\n"); return 2; }
    std::vector<int> w(n + 1);
    for (int l = 0; l <= n; ++l) w[l] = atoi(argv[5 + l]);
    std::vector<float> x = read_bin(dir + "/x.bin", (size_t)B * w[0]);
    std::vector<std::vector<float>> C(n);
    // 16-byte aligned, exact-size heap buffers for the coefficients (the fused kernel uses vector loads)
    std::vector<float*> Cp(n), act(n + 1);
    for (int l = 0; l < n; ++l) {
        const size_t cnt = (size_t)w[l] * w[l + 1] * (d + 1);
        C[l] = read_bin(dir + "/C" + std::to_string(l) + ".bin", cnt);
        Cp[l] = (float*)aligned_alloc(16, (cnt * 4 + 15) / 16 * 16);
        for (size_t i = 0; i < cnt; ++i) Cp[l][i] = C[l][i];
    }
    act[0] = x.data();
    for (int l = 1; l <= n; ++l) {
        act[l] = (float*)malloc(sizeof(float) * B * w[l]);
        for (size_t i = 0; i < (size_t)B * w[l]; ++i) act[l][i] = NAN;
    }
    const size_t wn = chebykan_stack_workspace_bytes(B, n, w.data(), d);
    float* ws = wn ? (float*)malloc(wn) : nullptr;
    const int rc = chebykan_stack_forward(n, w.data(), d, B, Cp.data(), act.data(), ws, wn, nullptr);
    if (rc != CHEBYKAN_OK) { fprintf(stderr, "stack forward: %s\n", chebykan_status_string((chebykan_status)rc)); return 1; }
    auto dump = [&](const std::string& name, const float* p, size_t cnt) {
        FILE* f = fopen((dir + "/" + name).c_str(), "wb");
        if (!f || fwrite(p, sizeof(float), cnt, f) != cnt) { fprintf(stderr, "cannot write %s\n", name.c_str()); exit(3); }
        fclose(f);
    };
    // backward through the same stack
    std::vector<float> dy = read_bin(dir + "/dy.bin", (size_t)B * w[n]);
    std::vector<float*> grad(n + 1), dC(n);
    grad[n] = dy.data();
    for (int l = 0; l < n; ++l) {
        grad[l] = (float*)malloc(sizeof(float) * B * w[l]);
        for (size_t i = 0; i < (size_t)B * w[l]; ++i) grad[l][i] = NAN;
        const size_t cnt = (size_t)w[l] * w[l + 1] * (d + 1);
        dC[l] = (float*)malloc(sizeof(float) * cnt);
        for (size_t i = 0; i < cnt; ++i) dC[l][i] = NAN;
    }
    const int rb = chebykan_stack_backward(n, w.data(), d, B, Cp.data(), act.data(), grad.data(), dC.data(), ws, wn, nullptr);
    if (rb != CHEBYKAN_OK) { fprintf(stderr, "stack backward: %s\n", chebykan_status_string((chebykan_status)rb)); return 1; }
    for (int l = 0; l < n; ++l) {
        dump("g" + std::to_string(l) + ".bin", grad[l], (size_t)B * w[l]);
        dump("dC" + std::to_string(l) + ".bin", dC[l], (size_t)w[l] * w[l + 1] * (d + 1));
        free(grad[l]);
        free(dC[l]);
    }
    for (int l = 1; l <= n; ++l) {
        dump("y" + std::to_string(l - 1) + ".bin", act[l], (size_t)B * w[l]);
        free(act[l]);
    }
    for (int l = 0; l < n; ++l) free(Cp[l]);
    free(ws);
    return 0;
}
