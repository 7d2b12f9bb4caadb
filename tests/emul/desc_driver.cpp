// Driver of tests/test_desc.py: runs the kernels GENERATED for one descriptor on the CPU.
// The generated source (-DGEN_SRC="file") is compiled as plain C++ against the host stand-in of
// the HIP runtime, with AddressSanitizer; the kernels have no barriers or cross-lane operations,
// so a launch run as nested loops computes exactly what the GPU computes.
//   argv: dir count box order nruns last_dim   (dir holds table.i32, bc.f32 [count], c.f32 [box])
//   writes list.i32 [count*order], thp.f32 [count], expand.f32 [box] (expansion of bc.f32)
#include <hip/hip_runtime.h>
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
    wr(dir + "/list.i32", list);
    wr(dir + "/thp.f32", thp);
    wr(dir + "/expand.f32", ex);
    printf("rc=0\n");
    return 0;
}
