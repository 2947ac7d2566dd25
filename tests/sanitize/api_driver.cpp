// Host-side validation of the C-ABI entry points under the address / undefined-behaviour sanitizers.
// Built by tests/test_sanitizers.py from paper_2505_14969_amd/csrc/api.hip (host pass only) and this
// file, whose stand-ins for the kernel launchers count their calls: every call below must be turned
// down (or found empty) by the validation, so no launcher is ever reached and no GPU is needed.
#include <cstdio>
#include <cstring>

#include "../../paper_2505_14969_amd/csrc/launch.hpp"

static int launches = 0;
namespace stree {
hipError_t launch_tree_index(const stree_dims &, const int32_t *, int32_t *, uint32_t *, int32_t *, int32_t *, hipStream_t) { ++launches; return hipSuccess; }
hipError_t launch_tree_conv(const stree_dims &, const int32_t *, const void *, const void *, const void *, const void *, void *, int32_t *, hipStream_t) { ++launches; return hipSuccess; }
hipError_t launch_tree_conv_replay(const stree_dims &, int, const int32_t *, const int32_t *, const void *, const int32_t *, const void *, const void *, const void *, const void *, void *, void *, int32_t *, int32_t *, hipStream_t) { ++launches; return hipSuccess; }
hipError_t launch_tree_ssd_fma(const stree_dims &, const int32_t *, const void *, const float *, const float *, const void *, const void *, const float *, const void *, void *, int32_t *, hipStream_t) { ++launches; return hipSuccess; }
bool tree_ssd_mfma_supported(const stree_dims &, const void *, const void *, const void *, const void *, const void *) { return true; }
hipError_t launch_tree_ssd_mfma(const stree_dims &, const int32_t *, const void *, const float *, const float *, const void *, const void *, const float *, const void *, void *, int32_t *, hipStream_t) { ++launches; return hipSuccess; }
bool tree_ssd_replay_fused_supported(const stree_dims &, const stree_dims &, const void *, const void *, const void *, const void *, const void *, const void *, const void *, const void *) { return true; }
hipError_t launch_tree_ssd_replay_fused(const stree_dims &, const stree_dims &, const int32_t *, const int32_t *, const void *, const float *, const void *, const int32_t *, const void *, const float *, const float *, const void *, const void *, const float *, const void *, void *, void *, int32_t *, int32_t *, hipStream_t) { ++launches; return hipSuccess; }
bool linear_ssd_supported(const stree_dims &d, const void *, const void *, const void *, const void *, const void *, const void *) { return d.headdim == 64; }
hipError_t launch_linear_ssd(const stree_dims &, const void *, const float *, const float *, const void *, const void *, const float *, const void *, void *, void *, hipStream_t) { ++launches; return hipSuccess; }
hipError_t prepare_tree_ssd_mfma() { return hipSuccess; }
hipError_t prepare_tree_ssd_fma() { return hipSuccess; }
hipError_t launch_gate_norm(const stree_dims &, const void *, const void *, long, const void *, float, void *, hipStream_t) { ++launches; return hipSuccess; }
hipError_t launch_commit_state(const stree_dims &, const int32_t *, const int32_t *, const void *, const float *, const float *, const void *, const void *, void *, const void *, const void *, void *, int32_t *, hipStream_t) { ++launches; return hipSuccess; }
}  // namespace stree

static int fails = 0;
#define EXPECT(call, want)                                                               \
    do {                                                                                 \
        const long got_ = (long)(call);                                                  \
        if (got_ != (long)(want)) { printf("line %d: got %ld, want %ld\n", __LINE__, got_, (long)(want)); ++fails; } \
    } while (0)

int main() {
    alignas(16) char buf[64];
    void *p = buf;                       // never dereferenced by the validation
    const int32_t *ip = reinterpret_cast<const int32_t *>(buf);
    const float *fp = reinterpret_cast<const float *>(buf);
    float *fo = reinterpret_cast<float *>(buf);
    stree_dims ok = {2, 64, 8, 64, 128, 1, 4, STREE_BF16, STREE_F32, 0, 0, 0, 0};
    stree_dims d = ok;
    EXPECT(stree_workspace_bytes(&ok), 0);
    EXPECT(stree_prepare(), STREE_OK);
    EXPECT(stree_workspace_bytes(nullptr), (size_t)-1);
    d = ok; d.nnodes = 257; EXPECT(stree_workspace_bytes(&d), (size_t)-1);
    EXPECT(stree_tree_ssd(nullptr, ip, p, fp, fp, p, p, nullptr, nullptr, p, nullptr, nullptr), STREE_ERR_NULL_ARG);
    EXPECT(stree_tree_ssd(&ok, ip, nullptr, fp, fp, p, p, nullptr, nullptr, p, nullptr, nullptr), STREE_ERR_NULL_ARG);
    d = ok; d.ngroups = 3; EXPECT(stree_tree_ssd(&d, ip, p, fp, fp, p, p, nullptr, nullptr, p, nullptr, nullptr), STREE_ERR_BAD_SHAPE);
    d = ok; d.io_dtype = 9; EXPECT(stree_tree_ssd(&d, ip, p, fp, fp, p, p, nullptr, nullptr, p, nullptr, nullptr), STREE_ERR_BAD_DTYPE);
    d = ok; d.x_stride_n = 8; EXPECT(stree_tree_ssd(&d, ip, p, fp, fp, p, p, nullptr, nullptr, p, nullptr, nullptr), STREE_ERR_BAD_STRIDE);
    d = ok; d.x_stride_n = 1LL << 28;                             // 64 nodes x 2^28 elements: beyond 32-bit offsets
    EXPECT(stree_tree_ssd(&d, ip, p, fp, fp, p, p, nullptr, nullptr, p, nullptr, nullptr), STREE_ERR_BAD_STRIDE);
    d = ok; d.batch = 65535; d.nnodes = 256; d.nheads = 65535;    // dt index beyond 32 bits
    EXPECT(stree_tree_ssd(&d, ip, p, fp, fp, p, p, nullptr, nullptr, p, nullptr, nullptr), STREE_ERR_BAD_SHAPE);
    d = ok; d.state_dtype = 9; EXPECT(stree_tree_ssd(&d, ip, p, fp, fp, p, p, nullptr, nullptr, p, nullptr, nullptr), STREE_ERR_BAD_DTYPE);
    d = ok; d.io_dtype = STREE_F32; d.state_dtype = STREE_BF16;   // a bf16 state goes with bf16 io only
    EXPECT(stree_tree_ssd(&d, ip, p, fp, fp, p, p, nullptr, nullptr, p, nullptr, nullptr), STREE_ERR_BAD_DTYPE);
    d = ok; d.state_dtype = STREE_BF16;                           // a bf16 state starts on a 16-byte boundary
    EXPECT(stree_tree_ssd(&d, ip, p, fp, fp, p, p, nullptr, buf + 2, p, nullptr, nullptr), STREE_ERR_BAD_SHAPE);
    EXPECT(stree_commit_state(&d, ip, ip, p, fp, fp, p, nullptr, buf + 8, nullptr, nullptr, nullptr, nullptr, nullptr), STREE_ERR_BAD_SHAPE);
    d = ok; d.flags = STREE_FLAG_DT_SOFTPLUS;                     // the softplus needs its bias vector
    EXPECT(stree_tree_ssd(&d, ip, p, fp, fp, p, p, nullptr, nullptr, p, nullptr, nullptr), STREE_ERR_NULL_ARG);
    d = ok; d.batch = 0; EXPECT(stree_tree_ssd(&d, ip, p, fp, fp, p, p, nullptr, nullptr, p, nullptr, nullptr), STREE_OK);
    d = ok; d.conv_width = 5; EXPECT(stree_tree_conv(&d, ip, p, p, p, nullptr, p, nullptr, nullptr), STREE_ERR_BAD_SHAPE);
    EXPECT(stree_tree_conv(&ok, ip, p, p, p, nullptr, nullptr, nullptr, nullptr), STREE_ERR_NULL_ARG);
    EXPECT(stree_commit_state(&ok, ip, nullptr, p, fp, fp, p, nullptr, fo, nullptr, nullptr, nullptr, nullptr, nullptr), STREE_ERR_NULL_ARG);
    EXPECT(stree_commit_state(&ok, ip, ip, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr), STREE_ERR_NULL_ARG);
    d = ok; d.dstate = 30; EXPECT(stree_commit_state(&d, ip, ip, p, fp, fp, p, nullptr, fo, nullptr, nullptr, nullptr, nullptr, nullptr), STREE_ERR_BAD_SHAPE);
    d = ok; d.nnodes = 300; EXPECT(stree_tree_index(&d, ip, nullptr, nullptr, nullptr, nullptr, nullptr), STREE_ERR_BAD_SHAPE);
    stree_replay prev;
    memset(&prev, 0, sizeof prev);
    prev.nnodes = 64; prev.parent = ip; prev.accepted = ip; prev.x = p; prev.dt = fp; prev.Bm = p;
    EXPECT(stree_tree_ssd_replay(&ok, nullptr, ip, p, fp, fp, p, p, nullptr, fp, fo, p, nullptr, nullptr, nullptr), STREE_ERR_NULL_ARG);
    EXPECT(stree_tree_ssd_replay(&ok, &prev, ip, p, fp, fp, p, p, nullptr, nullptr, fo, p, nullptr, nullptr, nullptr), STREE_ERR_NULL_ARG);
    prev.nnodes = 0; EXPECT(stree_tree_ssd_replay(&ok, &prev, ip, p, fp, fp, p, p, nullptr, fp, fo, p, nullptr, nullptr, nullptr), STREE_ERR_BAD_SHAPE);
    prev.nnodes = 64; prev.x_stride_n = 8; EXPECT(stree_tree_ssd_replay(&ok, &prev, ip, p, fp, fp, p, p, nullptr, fp, fo, p, nullptr, nullptr, nullptr), STREE_ERR_BAD_STRIDE);
    prev.x_stride_n = 0;
    EXPECT(stree_tree_conv_replay(&ok, &prev, nullptr, ip, p, p, p, nullptr, p, p, nullptr, nullptr, nullptr), STREE_ERR_NULL_ARG);
    // one buffer as this step's conv output and the previous step's: caught before anything is launched
    EXPECT(stree_tree_step(&ok, &prev, p, ip, p, p, p, nullptr, p, p, fp, fp, nullptr, fp, fo, p, nullptr, nullptr, nullptr), STREE_ERR_BAD_ALIAS);
    d = ok; d.batch = 0; EXPECT(stree_tree_step(&d, &prev, p, ip, p, p, p, nullptr, p, p, fp, fp, nullptr, fp, fo, p, nullptr, nullptr, nullptr), STREE_OK);
    d = ok; d.headdim = 32; d.nnodes = 4096; EXPECT(stree_linear_ssd(&d, p, fp, fp, p, p, nullptr, nullptr, p, fo, nullptr), STREE_ERR_BAD_SHAPE);
    d = ok; d.nnodes = 1 << 25; EXPECT(stree_linear_ssd(&d, p, fp, fp, p, p, nullptr, nullptr, p, fo, nullptr), STREE_ERR_BAD_SHAPE);
    EXPECT(stree_linear_ssd(&ok, p, fp, fp, p, nullptr, nullptr, nullptr, p, fo, nullptr), STREE_ERR_NULL_ARG);
    EXPECT(stree_gate_norm(&ok, p, p, 100, p, 1e-5f, p, nullptr), STREE_ERR_BAD_STRIDE);
    EXPECT(stree_gate_norm(&ok, p, nullptr, 0, p, 1e-5f, p, nullptr), STREE_ERR_NULL_ARG);
    EXPECT(stree_gate_norm(&ok, p, p, 0, p, -1.f, p, nullptr), STREE_ERR_BAD_SHAPE);
    for (int c = 0; c <= 7; ++c) EXPECT(stree_status_string(c) != nullptr && stree_status_string(c)[0] != 0, 1);
    EXPECT(launches, 0);
    printf("%d mismatches, %d launches\n", fails, launches);
    return fails != 0 || launches != 0;
}
