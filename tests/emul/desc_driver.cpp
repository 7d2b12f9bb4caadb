// Driver of tests/test_desc.py: runs the kernels GENERATED for one descriptor on the CPU.
// The generated source (-DGEN_SRC="file") is compiled as plain C++ against the host stand-in of
// the HIP runtime, with AddressSanitizer; the list, product and expansion kernels have no barriers or
// cross-lane operations, so a launch run as nested loops computes exactly what the GPU computes; the
// moment kernels are launched in a shape (one thread per block, one slice) for which that also holds.
//   argv: dir count box order nruns last_dim [N]  (dir holds table.i32, bc.f32 [count], c.f32 [box], x.f32 [N*n])
//   writes list.i32 [count*order], thp.f32 [count], expand.f32 [box] (expansion of bc.f32), moment.f32 [count],
//   sum_last.f32 [nruns] (every run of bc.f32 summed)
//   when dir holds gather.i32 ([g][order] dense positions; gather_scale.f32 [g] optional): gather.f32 [g]
//   when dir holds onto.f32 [box]: expand_onto.f32 [box], bc.f32 laid over it (only the elements the structure holds)
//   when dir holds mk_r.i32 (order 3): mttkrp.f32 [dim0][R] from mk_c.f32 [dim1][R] and mk_d.f32 [dim2][R]
#include <hip/hip_runtime.h>
// LDS of the generated moment kernels: the dynamic chunk buffer is a global here, static arrays keep their
// zero initialisation (the reduce kernel reads rows of its array that other threads of the block wrote)
extern "C" { float st_gen_lds[2 * 8192]; }
#define ST_DYN_LDS
#undef __shared__
#define __shared__ static
#include GEN_SRC
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

template <typename T> static std::vector<T> rd(const std::string &path, size_t n)
{
    std::vector<T> v(n ? n : 1);
    FILE *f = fopen(path.c_str(), "rb");
    if (!f || (n && fread(v.data(), sizeof(T), n, f) != n)) { fprintf(stderr, "cannot read %s\n", path.c_str()); exit(2); }
    fclose(f);
    v.resize(n);
    return v;
}
template <typename T> static void wr(const std::string &path, const std::vector<T> &v)
{
    FILE *f = fopen(path.c_str(), "wb");
    if (!f || (v.size() && fwrite(v.data(), sizeof(T), v.size(), f) != v.size())) { fprintf(stderr, "cannot write %s\n", path.c_str()); exit(2); }
    fclose(f);
}

int main(int argc, char **argv)
{
    if (argc < 7) return 2;
    const std::string dir = argv[1];
    const size_t count = (size_t)atol(argv[2]), box = (size_t)atol(argv[3]), order = (size_t)atol(argv[4]);
    const size_t nruns = (size_t)atol(argv[5]);
    if (count != (size_t)ST_COUNT || nruns != (size_t)ST_NRUNS || order != (size_t)ST_D) return 3;
    std::vector<int> tab = rd<int>(dir + "/table.i32", (size_t)ST_PREFIXES + nruns);
    std::vector<float> bc = rd<float>(dir + "/bc.f32", count), c = rd<float>(dir + "/c.f32", box);
    std::vector<int> list(count * order, -7);
    std::vector<float> thp(count, -7.f), ex(box, -7.f);
    const unsigned rb = (unsigned)((nruns + 3) / 4);
    if (rb) {
        hipLaunchKernelGGL(st_gen_list, dim3(rb), dim3(256), 0, 0, tab.data(), list.data());
        hipLaunchKernelGGL(st_gen_thp, dim3(rb), dim3(256), 0, 0, tab.data(), bc.data(), c.data(), thp.data());
    }
    const size_t last_dim = (size_t)atol(argv[6]), ethreads = last_dim % 4 == 0 ? box / 4 : box;   // as the library launches it
    hipLaunchKernelGGL(st_gen_expand, dim3((unsigned)((ethreads + 255) / 256)), dim3(256), 0, 0, tab.data(), bc.data(), ex.data());
#ifdef ST_NTILES
    // moment kernels: one thread per block and one sample slice, so that the missing barriers change nothing
    if (argc > 7) {
        const long long N = atol(argv[7]);
        std::vector<int> full = rd<int>(dir + "/table.i32", (size_t)ST_TILES_OFF + (size_t)ST_NTILES * ST_D);
        std::vector<float> X = rd<float>(dir + "/x.f32", (size_t)N * ST_DIM0), ws((size_t)ST_NTILES * 64, -7.f), sc(count, -7.f);
        int ch = 8192 / ST_MNP;
        ch = ch > 64 ? 64 : ch & ~3;
        const long long slice = (N + ch - 1) / ch * ch;
        hipLaunchKernelGGL(st_gen_moment, dim3(ST_NTILES), dim3(1), 0, 0, full.data(), X.data(), N, ch, slice, ws.data());
        hipLaunchKernelGGL(st_gen_moment_reduce, dim3((ST_NTILES * 64 + 15) / 16), dim3(256), 0, 0, full.data(), ws.data(), 1,
                           sc.data(), 0);
        wr(dir + "/moment.f32", sc);
    }
#endif
    if (FILE *f = fopen((dir + "/gather.i32").c_str(), "rb")) {
        fseek(f, 0, SEEK_END);
        const size_t g = (size_t)ftell(f) / (sizeof(int) * order);
        fclose(f);
        std::vector<int> idx = rd<int>(dir + "/gather.i32", g * order);
        std::vector<float> scale, out(g, -7.f);
        if (FILE *h = fopen((dir + "/gather_scale.f32").c_str(), "rb")) { fclose(h); scale = rd<float>(dir + "/gather_scale.f32", g); }
        std::vector<float> addend;
        if (FILE *h = fopen((dir + "/gather_addend.f32").c_str(), "rb")) { fclose(h); addend = rd<float>(dir + "/gather_addend.f32", g); }
        if (g) hipLaunchKernelGGL(st_gen_gather, dim3((unsigned)((g + 255) / 256)), dim3(256), 0, 0, tab.data(), bc.data(), idx.data(),
                                  (long long)g, (int)order, 0, scale.empty() ? (const float *)nullptr : scale.data(),
                                  addend.empty() ? (const float *)nullptr : addend.data(), out.data());
        wr(dir + "/gather.f32", out);
    }
    if (FILE *f = fopen((dir + "/onto.f32").c_str(), "rb")) {
        fclose(f);
        std::vector<float> onto = rd<float>(dir + "/onto.f32", box);
        hipLaunchKernelGGL(st_gen_expand_onto, dim3((unsigned)((box + 255) / 256)), dim3(256), 0, 0, tab.data(), bc.data(), onto.data());
        wr(dir + "/expand_onto.f32", onto);
    }
#if ST_D == 3
    // the generated MTTKRP, launched with one thread per workgroup (its sums over the threads of a workgroup need a
    // barrier): mk_r.i32 holds R, mk_c.f32 is [dim1][R], mk_d.f32 is [dim2][R]; writes mttkrp.f32 [dim0][R]
    if (FILE *f = fopen((dir + "/mk_r.i32").c_str(), "rb")) {
        fclose(f);
        const int R = rd<int>(dir + "/mk_r.i32", 1)[0];
        std::vector<float> Cm = rd<float>(dir + "/mk_c.f32", (size_t)ST_DIM1 * R), Dm = rd<float>(dir + "/mk_d.f32", (size_t)ST_DIM2 * R);
        std::vector<float> A((size_t)ST_DIM0 * R, -7.f);
        hipLaunchKernelGGL(st_gen_mttkrp, dim3(ST_DIM0, (unsigned)((R + 15) / 16)), dim3(1), 0, 0, tab.data(), bc.data(), Cm.data(),
                           Dm.data(), A.data(), R);
        wr(dir + "/mttkrp.f32", A);
        // the second half of the matrix-core route, when every run is a whole fibre (count = runs * dim2): Y(run, r)
        // = sum_l Bc(run, l) D(l, r) in plain loops here, then the generated combine kernel, one thread per workgroup
        if (nruns > 0 && count == nruns * (size_t)ST_DIM2) {
            std::vector<float> Y(nruns * (size_t)R, 0.f), A2((size_t)ST_DIM0 * R, -7.f);
            for (size_t run = 0; run < nruns; ++run)
                for (int r = 0; r < R; ++r) {
                    float acc = 0.f;
                    for (size_t l = 0; l < (size_t)ST_DIM2; ++l) acc += bc[run * ST_DIM2 + l] * Dm[l * R + r];
                    Y[run * R + r] = acc;
                }
            hipLaunchKernelGGL(st_gen_mttkrp_combine, dim3(ST_DIM0, (unsigned)((R + 63) / 64)), dim3(1), 0, 0, tab.data(), Y.data(),
                               Cm.data(), A2.data(), R);
            wr(dir + "/mttkrp_combine.f32", A2);
        }
    }
#endif
    {   // marginalization of the last variable, one thread per workgroup (its sum over the lanes needs a barrier)
        std::vector<float> sums(nruns ? nruns : 1, -7.f);
        if (nruns) hipLaunchKernelGGL(st_gen_sum_last, dim3((unsigned)nruns), dim3(1), 0, 0, tab.data(), bc.data(), sums.data());
        sums.resize(nruns);
        wr(dir + "/sum_last.f32", sums);
    }
    wr(dir + "/list.i32", list);
    wr(dir + "/thp.f32", thp);
    wr(dir + "/expand.f32", ex);
    printf("rc=0\n");
    return 0;
}
