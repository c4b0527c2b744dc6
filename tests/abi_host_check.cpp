// Host-side argument validation of the C ABI under AddressSanitizer + UndefinedBehaviorSanitizer (host code only; no GPU is touched:
// every call below must be refused before anything is enqueued).  Built and run by tests/test_abi.py::test_host_validation_under_sanitizers.
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "../include/sparseffn.h"

static int failures = 0;
#define EXPECT(call, code) do { int rc_ = (call); if (rc_ != (code)) { printf("FAIL line %d: %s -> %d, expected %d (%s)\n", __LINE__, #call, rc_, (code), sffn_last_error()); ++failures; } } while (0)

int main() {
    uint16_t* fake = (uint16_t*)0x1000;        // 16-byte aligned, never dereferenced
    uint8_t* fake8 = (uint8_t*)0x2000;
    uint16_t* odd = (uint16_t*)0x1008;
    float* fakef = (float*)0x3000;
    void* ws = (void*)0x4000;
    EXPECT(prune24_compress(nullptr, 64, 64, 64, 0, 0, fake, fake8, nullptr), SFFN_EINVAL);
    EXPECT(prune24_compress(fake, 64, 60, 64, 0, 0, fake, fake8, nullptr), SFFN_EINVAL);
    EXPECT(prune24_compress(fake, 64, 64, 32, 0, 0, fake, fake8, nullptr), SFFN_EINVAL);
    EXPECT(prune24_compress(odd, 64, 64, 64, 0, 0, fake, fake8, nullptr), SFFN_EINVAL);
    EXPECT(prune24_compress(fake, (int64_t)1 << 40, 64, 64, 0, 0, fake, fake8, nullptr), SFFN_EUNSUPPORTED);
    EXPECT(sqrelu_vnm_compress(fake, 64, 64, 64, 12, fake, fake8, fake8, nullptr), SFFN_EUNSUPPORTED);
    EXPECT(sqrelu_vnm_compress(fake, 64, 64, 64, 64, fake, fake8, fake8, nullptr), SFFN_EINVAL);
    EXPECT(spmm24_fwd(fake, fake, fake8, nullptr, 64, 64, 65, fake, nullptr), SFFN_EINVAL);
    EXPECT(spmm24_dgrad(fake, fake, nullptr, 64, 64, 64, fake, nullptr), SFFN_EINVAL);
    EXPECT(vnm_spmm(fake, fake8, fake8, fake, 64, 0, 64, 64, 64, 64, 8, fake, nullptr, 0, nullptr), SFFN_EWORKSPACE);
    EXPECT(vnm_spmm(fake, fake8, fake8, fake, 192, 0, (int64_t)1 << 20, 64, 192, 64, 16, fake, ws, (size_t)1 << 40, nullptr), SFFN_EUNSUPPORTED);   // plain-2:4 route (4 * 192 / 16 is not a multiple of 64): T below 65536
    EXPECT(dsqrelu_vnm(fake, fake, fake8, fake8, 64, 100, 64, 8, fake, nullptr), SFFN_EINVAL);
    EXPECT(vnm_wgrad(fake, fake8, fake8, fake, 64, 64, 64, 64, 8, 0, fake, ws, 16, nullptr), SFFN_EWORKSPACE);
    EXPECT(quantize_fp8(fake, 12, 1.0f, fake8, nullptr, nullptr), SFFN_EINVAL);
    EXPECT(quantize_fp8(fake, 16, 0.0f, fake8, nullptr, nullptr), SFFN_EINVAL);
    EXPECT(quantize_fp8(fake, 16, -1.0f, fake8, nullptr, nullptr), SFFN_EINVAL);
    EXPECT(prune24_compress_fp8(fake, 64, 64, 64, 0, 3, 1.0f, fake8, fake8, nullptr, nullptr), SFFN_EINVAL);
    EXPECT(spmm24_fp8(fake8, 1.0f, fake8, fake8, 1.0f, nullptr, 64, 64, 64, fake, nullptr), SFFN_EINVAL);        // K must be a multiple of 128
    EXPECT(vnm_spmm_fp8(fake8, fake8, fake8, 1.0f, fake8, 1.0f, 0, 64, 64, 128, 64, 8, fake, ws, 16, nullptr), SFFN_EWORKSPACE);
    sffn_cfg cfg;
    memset(&cfg, 0, sizeof(cfg));
    cfg.T = 512; cfg.D = 256; cfg.F = 1024; cfg.V = 64; cfg.M = 8;
    sffn_ws_layout lay;
    EXPECT(sffn_workspace_layout(&cfg, &lay), SFFN_OK);
    if (lay.total != sffn_workspace_bytes(&cfg) || lay.total == 0) { printf("FAIL: layout total\n"); ++failures; }
    EXPECT(sffn_workspace_layout(&cfg, nullptr), SFFN_EINVAL);
    EXPECT(sffn_workspace_layout(nullptr, &lay), SFFN_EINVAL);
    EXPECT(ffn_sparse_step(&cfg, fake, fake, fake, fakef, fake, fake, fake, fake, fake, ws, 16, nullptr), SFFN_EWORKSPACE);
    EXPECT(ffn_sparse_step(nullptr, fake, fake, fake, fakef, fake, fake, fake, fake, fake, ws, (size_t)1 << 40, nullptr), SFFN_EINVAL);
    cfg.M = 12;
    EXPECT(ffn_sparse_step(&cfg, fake, fake, fake, fakef, fake, fake, fake, fake, fake, ws, (size_t)1 << 40, nullptr), SFFN_EUNSUPPORTED);
    if (sffn_workspace_bytes(&cfg) != 0) { printf("FAIL: unknown M must have no layout\n"); ++failures; }
    cfg.M = 8;
    int64_t seg_bad[3] = {0, 100, 512}, seg_ok[3] = {0, 320, 512}, seg_many[70];
    memset(seg_many, 0, sizeof(seg_many));
    EXPECT(ffn_sparse_step_grouped(&cfg, 2, seg_bad, fake, fake, fake, fakef, fake, fake, fake, fake, fake, ws, (size_t)1 << 40, nullptr), SFFN_EINVAL);
    EXPECT(ffn_sparse_step_grouped(&cfg, 2, seg_ok, fake, fake, fake, fakef, fake, fake, fake, fake, fake, ws, 16, nullptr), SFFN_EWORKSPACE);
    EXPECT(ffn_sparse_step_grouped(&cfg, 65, seg_many, fake, fake, fake, fakef, fake, fake, fake, fake, fake, ws, (size_t)1 << 40, nullptr), SFFN_EINVAL);
    EXPECT(ffn_sparse_step_grouped(&cfg, 2, nullptr, fake, fake, fake, fakef, fake, fake, fake, fake, fake, ws, (size_t)1 << 40, nullptr), SFFN_EINVAL);
    // Alg. 1 / Alg. 2 as separate calls on three buffers: sizes, alignment, overlap, the pointers each half needs, the flags
    sffn_buffers sz;
    EXPECT(sffn_buffer_sizes(&cfg, 1, &sz), SFFN_OK);
    if (sz.scratch_bytes + sz.saved_bytes + sz.weights_bytes != sffn_workspace_bytes(&cfg) || sz.scratch != nullptr) { printf("FAIL: buffer sizes\n"); ++failures; }
    EXPECT(sffn_buffer_sizes(&cfg, 1, nullptr), SFFN_EINVAL);
    const uintptr_t far = (uintptr_t)1 << 40;
    sffn_buffers good = {(void*)far, sz.scratch_bytes, (void*)(2 * far), sz.saved_bytes, (void*)(3 * far), sz.weights_bytes};
    sffn_buffers shorter = good, crossing = good, skewed = good;
    shorter.weights_bytes -= 256;
    crossing.saved = (void*)(far + sz.scratch_bytes - 256);
    skewed.scratch = (void*)(far + 64);
    EXPECT(ffn_sparse_forward(&cfg, fake, fake, fake, fakef, fake, &shorter, nullptr), SFFN_EWORKSPACE);
    EXPECT(ffn_sparse_forward(&cfg, fake, fake, fake, fakef, fake, &crossing, nullptr), SFFN_EINVAL);
    EXPECT(ffn_sparse_forward(&cfg, fake, fake, fake, fakef, fake, &skewed, nullptr), SFFN_EINVAL);
    EXPECT(ffn_sparse_forward(&cfg, fake, fake, nullptr, fakef, fake, &good, nullptr), SFFN_EINVAL);
    EXPECT(ffn_sparse_backward(&cfg, fake, fake, fake, fake, nullptr, &good, nullptr), SFFN_EINVAL);
    EXPECT(ffn_sparse_backward(&cfg, fake, fake, fake, fake, fake, nullptr, nullptr), SFFN_EINVAL);
    cfg.flags = 64;
    EXPECT(ffn_sparse_forward(&cfg, fake, fake, fake, fakef, fake, &good, nullptr), SFFN_EINVAL);                       // unknown flag
    cfg.flags = 0;
    sffn_buffers sz8;
    EXPECT(sffn_fp8_buffer_sizes(&cfg, 1, &sz8), SFFN_OK);
    sffn_fp8_scales sc8 = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f};
    sffn_buffers good8 = {(void*)far, sz8.scratch_bytes, (void*)(2 * far), sz8.saved_bytes, (void*)(3 * far), sz8.weights_bytes};
    EXPECT(ffn_sparse_backward_fp8(&cfg, &sc8, fake, fake, fake, nullptr, &good8, nullptr, nullptr), SFFN_EINVAL);
    good8.saved_bytes -= 256;
    EXPECT(ffn_sparse_forward_fp8(&cfg, &sc8, fake, fake, fake, fakef, fake, &good8, nullptr, nullptr), SFFN_EWORKSPACE);
    sffn_cfg big = cfg;
    big.T = 2048; big.D = 1024; big.F = 4096;
    EXPECT(ffn_sparse_step_noalloc(&big, fake, fake, fake, fakef, fake, fake, fake, fake, fake, nullptr), SFFN_EWORKSPACE);
    // router: host segment table and capacity checks
    sffn_cfg r = cfg;
    r.T = 100; r.D = 64; r.F = 1024; r.M = 16;
    int64_t rs_ok[5] = {0, 64, 128, 128, 192}, rs_over[5] = {0, 64, 128, 256, 448};
    int32_t* fake32 = (int32_t*)0x5000;
    EXPECT(ffn_router_step(&r, rs_ok, fake32, fake, fake, fake, fakef, fake, fake, fake, fake, fake, ws, 16, nullptr), SFFN_EWORKSPACE);
    EXPECT(ffn_router_step(&r, rs_over, fake32, fake, fake, fake, fakef, fake, fake, fake, fake, fake, ws, (size_t)1 << 40, nullptr), SFFN_EINVAL);
    EXPECT(ffn_router_full_step(&r, fake, fake, fake, nullptr, fakef, fake, fake, fake, fake, fake, ws, (size_t)1 << 40, nullptr), SFFN_EINVAL);   // W2 missing: refused before the routing kernels
    EXPECT(venom_route(fake, fake, 100, 60, 16, fake32, fake32, fake32, fake32, nullptr, ws, (size_t)1 << 20, nullptr), SFFN_EINVAL);
    if (sffn_venom_rows(100, 16) != 128 + 256) { printf("FAIL: sffn_venom_rows\n"); ++failures; }
    printf(failures ? "abi_host_check: %d failure(s)\n" : "abi_host_check: all argument checks behave, no sanitizer report\n", failures);
    return failures ? 1 : 0;
}
