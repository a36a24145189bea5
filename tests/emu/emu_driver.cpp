// Host driver for the CPU emulation build of the library: reads raw fp32 inputs,
// calls the C ABI (whose launches now run on OS threads), writes raw outputs.
//   emu_driver <dir> <B> <I> <O> <degree> <family> [lut_size [basis]]
// <dir> holds x.bin, C.bin, dy.bin (and lut.bin when lut_size is given: the table-interpolated
// entry points are called then; basis 1..3 with lut_size 0 calls the Legendre / Hermite / Fourier entry
// points; basis 9 with a lut_size also reads dlut.bin and takes dx from the auxiliary derivative table);
// y.bin, dx.bin, dC.bin are written there.
#include <stdio.h>
#include <stdlib.h>
#include <math.h>
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

static void write_bin(const std::string& path, const float* p, size_t n)
{
    FILE* f = fopen(path.c_str(), "wb");
    if (!f || fwrite(p, sizeof(float), n, f) != n) { fprintf(stderr, "cannot write %s\n", path.c_str()); exit(3); }
    fclose(f);
}

int main(int argc, char** argv)
{
    if (argc < 7 || argc > 9) { fprintf(stderr, "usage: emu_driver dir B I O degree family [lut_size [basis]]\n"); return 2; }
    const int lut_size = argc >= 8 ? atoi(argv[7]) : 0;
    const int basis = argc >= 9 ? atoi(argv[8]) : 0;
    const std::string dir = argv[1];
    const long B = atol(argv[2]);
    const int I = atoi(argv[3]), O = atoi(argv[4]), d = atoi(argv[5]), family = atoi(argv[6]);
    const size_t K = d + 1;
    // exact-size heap buffers: AddressSanitizer sees any access past their ends
    std::vector<float> x = read_bin(dir + "/x.bin", (size_t)B * I);
    std::vector<float> C = read_bin(dir + "/C.bin", (size_t)I * O * K);
    std::vector<float> dy = read_bin(dir + "/dy.bin", (size_t)B * O);
    float* y = (float*)malloc(sizeof(float) * B * O);
    float* dx = (float*)malloc(sizeof(float) * B * I);
    float* dC = (float*)malloc(sizeof(float) * I * O * K);
    for (size_t i = 0; i < (size_t)B * O; ++i) y[i] = NAN;
    for (size_t i = 0; i < (size_t)B * I; ++i) dx[i] = NAN;
    for (size_t i = 0; i < (size_t)I * O * K; ++i) dC[i] = NAN;
    chebykan_set_kernel_family(family);
    const size_t wf = chebykan_workspace_bytes(B, I, O, d, CHEBYKAN_PASS_FORWARD);
    const size_t wb = chebykan_workspace_bytes(B, I, O, d, CHEBYKAN_PASS_BACKWARD);
    const size_t wn = wf > wb ? wf : wb;
    float* ws = wn ? (float*)malloc(wn) : nullptr;
    for (size_t i = 0; i < wn / 4; ++i) ws[i] = NAN;
    std::vector<float> lut;
    if (lut_size > 0) lut = read_bin(dir + "/lut.bin", K * (size_t)lut_size);
    std::vector<float> dlut;
    if (lut_size > 0 && basis == 9) dlut = read_bin(dir + "/dlut.bin", K * (size_t)lut_size);
    int rc = lut_size > 0 ? chebykan_forward_lut(x.data(), C.data(), lut.data(), lut_size, y, B, I, O, d, ws, wn, nullptr)
                          : chebykan_forward_basis(basis, x.data(), C.data(), y, B, I, O, d, ws, wn, nullptr);
    if (rc != CHEBYKAN_OK) { fprintf(stderr, "forward: %s\n", chebykan_status_string((chebykan_status)rc)); return 1; }
    rc = lut_size > 0 ? (basis == 9 ? chebykan_backward_lut2(x.data(), C.data(), dy.data(), lut.data(), dlut.data(), lut_size,
                                                             dx, dC, B, I, O, d, ws, wn, nullptr)
                                    : chebykan_backward_lut(x.data(), C.data(), dy.data(), lut.data(), lut_size, dx, dC, B, I,
                                                            O, d, ws, wn, nullptr))
                      : chebykan_backward_basis(basis, x.data(), C.data(), dy.data(), dx, dC, B, I, O, d, ws, wn, nullptr);
    if (rc != CHEBYKAN_OK) { fprintf(stderr, "backward: %s\n", chebykan_status_string((chebykan_status)rc)); return 1; }
    write_bin(dir + "/y.bin", y, (size_t)B * O);
    write_bin(dir + "/dx.bin", dx, (size_t)B * I);
    write_bin(dir + "/dC.bin", dC, (size_t)I * O * K);
    printf("workspace %zu bytes\n", wn);
    free(y); free(dx); free(dC); free(ws);
    return 0;
}
