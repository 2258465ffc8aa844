// Drives the C ABI's host half (argument validation, layout, pointer-table bookkeeping, launch sequencing) with
// stand-in launchers, under AddressSanitizer and UndefinedBehaviorSanitizer.  "Device" pointers are host buffers
// nobody dereferences (the stand-in kernels do nothing); the workspace is a host buffer the tables are written to.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "compactfusion.h"

extern std::vector<std::string> g_launch_log;
extern bool g_capturing;

static int g_failed = 0;
#define EXPECT(cond)                                                                    \
    do {                                                                                \
        if (!(cond)) { std::printf("line %d: %s\n", __LINE__, #cond); ++g_failed; }     \
    } while (0)

static std::string joined()
{
    std::string s;
    for (auto &k : g_launch_log) s += k + " ";
    g_launch_log.clear();
    return s;
}

// the call brought pointers to the table: by a launch of its own, or inside the single pass's first kernel
static bool uploaded(const std::string &seq) { return seq.find("k_upload_ptrs") != std::string::npos || seq.find("ptrs_in_reset") != std::string::npos; }

static cf_tensor_desc desc(int64_t n, int64_t c, int dt, int bits, int scale, int group = 128)
{
    cf_tensor_desc d;
    d.n_tokens = n; d.n_channels = c; d.dtype = dt; d.bits = bits; d.scale = scale; d.group = group;
    return d;
}

struct Buffers {       // one tensor's buffers, sized by cf_sizes, 256-byte aligned
    void *x = nullptr, *recon = nullptr, *err = nullptr, *codes = nullptr, *scales = nullptr;
    size_t cb = 0, sb = 0, rb = 0, eb = 0;
    Buffers(const cf_tensor_desc &d, const cf_options *o)
    {
        EXPECT(cf_sizes(&d, o, &cb, &sb, &rb, &eb) == CF_OK);
        auto get = [](size_t n) { void *p = nullptr; if (posix_memalign(&p, 256, n ? n : 256) != 0) std::abort(); return p; };
        x = get(rb); recon = get(rb); err = get(eb); codes = get(cb); scales = get(sb);
    }
    ~Buffers() { std::free(x); std::free(recon); std::free(err); std::free(codes); std::free(scales); }
};

int main()
{
    // ---- descriptors and options
    size_t a = 0, b = 0, c = 0, e = 0;
    cf_tensor_desc good = desc(4096, 3072, CF_BF16, 1, CF_SCALE_CHANNEL);
    EXPECT(cf_sizes(&good, nullptr, &a, &b, &c, &e) == CF_OK && a == 4096u * 384 && b == 3072u * 4 && c == 4096u * 3072 * 2 && e == 4096u * 3072 * 4);
    EXPECT(cf_sizes(nullptr, nullptr, &a, &b, &c, &e) == CF_ERR_INVALID_ARG);
    cf_tensor_desc bad = desc(0, 3072, CF_BF16, 1, CF_SCALE_CHANNEL);
    EXPECT(cf_sizes(&bad, nullptr, &a, nullptr, nullptr, nullptr) == CF_ERR_SHAPE);
    bad = desc(16, 100, CF_BF16, 1, CF_SCALE_CHANNEL);
    EXPECT(cf_sizes(&bad, nullptr, &a, nullptr, nullptr, nullptr) == CF_ERR_SHAPE);
    bad = desc(16, 128, CF_BF16, 3, CF_SCALE_CHANNEL);
    EXPECT(cf_sizes(&bad, nullptr, &a, nullptr, nullptr, nullptr) == CF_ERR_UNSUPPORTED);
    bad = desc(16, 128, CF_BF16, 2, CF_SCALE_GROUP);
    EXPECT(cf_sizes(&bad, nullptr, &a, nullptr, nullptr, nullptr) == CF_ERR_UNSUPPORTED);
    bad = desc(16, 192, CF_BF16, 4, CF_SCALE_GROUP);
    EXPECT(cf_sizes(&bad, nullptr, &a, nullptr, nullptr, nullptr) == CF_ERR_SHAPE);
    bad = desc(16, 128, 7, 2, CF_SCALE_CHANNEL);
    EXPECT(cf_sizes(&bad, nullptr, &a, nullptr, nullptr, nullptr) == CF_ERR_UNSUPPORTED);
    cf_options o;
    std::memset(&o, 0, sizeof o);
    o.flags = 0x40;
    EXPECT(cf_sizes(&good, &o, &a, nullptr, nullptr, nullptr) == CF_ERR_UNSUPPORTED);
    o.flags = 0; o.ef = 9;
    EXPECT(cf_workspace_bytes(&good, 1, &o) == 0);
    o.ef = CF_EF_RECON;
    EXPECT(cf_workspace_bytes(&good, 0, &o) == 0 && cf_workspace_bytes(nullptr, 1, &o) == 0);
    EXPECT(std::strlen(cf_status_string(CF_ERR_WORKSPACE)) > 0 && std::strlen(cf_status_string((cf_status)99)) > 0);

    // ---- a mixed context: every compressor kind, ragged shapes
    std::vector<cf_tensor_desc> descs = {desc(1500, 1096, CF_BF16, 1, CF_SCALE_CHANNEL), desc(700, 520, CF_F32, 2, CF_SCALE_CHANNEL),
                                         desc(300, 384, CF_BF16, 4, CF_SCALE_GROUP, 128), desc(130, 1096, CF_BF16, 2, CF_SPARSE_NM, 8),
                                         desc(67, 3072, CF_BF16, 2, CF_SPARSE_NM, 16), desc(203, 1024, CF_BF16, 1, CF_LOWRANK, 32),
                                         desc(1, 8, CF_F32, 4, CF_SCALE_CHANNEL)};
    const int n = (int)descs.size();
    for (uint32_t flags : {0u, (uint32_t)CF_FLAG_SINGLE_PASS, (uint32_t)CF_FLAG_TWO_KERNEL, (uint32_t)(CF_FLAG_SINGLE_PASS | CF_FLAG_FIXED_GRID),
                           (uint32_t)CF_FLAG_LOWRANK_INT4}) {
        std::memset(&o, 0, sizeof o);
        o.flags = flags;
        const size_t ws_bytes = cf_workspace_bytes(descs.data(), n, &o);
        EXPECT(ws_bytes > 0);
        void *ws = nullptr;
        if (posix_memalign(&ws, 256, ws_bytes) != 0) return 2;
        cf_ctx *ctx = nullptr;
        EXPECT(cf_init(&ctx, descs.data(), n, &o, nullptr, ws_bytes, nullptr) == CF_ERR_WORKSPACE && ctx == nullptr);
        EXPECT(cf_init(&ctx, descs.data(), n, &o, (char *)ws + 16, ws_bytes, nullptr) == CF_ERR_WORKSPACE);
        EXPECT(cf_init(&ctx, descs.data(), n, &o, ws, ws_bytes - 1, nullptr) == CF_ERR_WORKSPACE);
        EXPECT(cf_init(nullptr, descs.data(), n, &o, ws, ws_bytes, nullptr) == CF_ERR_INVALID_ARG);
        EXPECT(cf_init(&ctx, descs.data(), n, &o, ws, ws_bytes, nullptr) == CF_OK && ctx != nullptr);
        g_launch_log.clear();

        std::vector<Buffers *> buf;
        std::vector<const void *> x;
        std::vector<void *> recon, err, codes, scales;
        for (auto &d : descs) {
            buf.push_back(new Buffers(d, &o));
            x.push_back(buf.back()->x); recon.push_back(buf.back()->recon); err.push_back(buf.back()->err);
            codes.push_back(buf.back()->codes); scales.push_back(buf.back()->scales);
        }
        // state errors, range errors, pointer errors: nothing may be launched
        EXPECT(cf_step_fused(ctx, 0, n, x.data(), recon.data(), err.data(), codes.data(), scales.data(), nullptr) == CF_ERR_STATE);
        EXPECT(cf_step_fused(ctx, 0, n + 1, x.data(), recon.data(), err.data(), codes.data(), scales.data(), nullptr) == CF_ERR_INVALID_ARG);
        EXPECT(cf_step_fused(ctx, -1, 1, x.data(), recon.data(), err.data(), codes.data(), scales.data(), nullptr) == CF_ERR_INVALID_ARG);
        EXPECT(cf_step_fused(nullptr, 0, n, x.data(), recon.data(), err.data(), codes.data(), scales.data(), nullptr) == CF_ERR_INVALID_ARG);
        EXPECT(cf_warmup(ctx, 0, n, nullptr, recon.data(), err.data(), nullptr) == CF_ERR_INVALID_ARG);
        EXPECT(joined().empty());
        EXPECT(cf_warmup(ctx, 0, n, x.data(), recon.data(), err.data(), nullptr) == CF_OK);
        EXPECT(joined().find("k_warmup") != std::string::npos);
        {   // overlapping and misaligned buffers
            std::vector<void *> r2 = recon;
            r2[0] = (char *)buf[0]->x + 256;                                    // inside x
            EXPECT(cf_step_fused(ctx, 0, n, x.data(), r2.data(), err.data(), codes.data(), scales.data(), nullptr) == CF_ERR_INVALID_ARG);
            r2 = recon; r2[1] = (char *)recon[1] + 4;                           // not 16-byte aligned
            EXPECT(cf_step_fused(ctx, 0, n, x.data(), r2.data(), err.data(), codes.data(), scales.data(), nullptr) == CF_ERR_INVALID_ARG);
            std::vector<void *> c2 = codes;
            c2[2] = (char *)buf[2]->err + buf[2]->eb - 16;                      // tail of err
            EXPECT(cf_step_fused(ctx, 0, n, x.data(), recon.data(), err.data(), c2.data(), scales.data(), nullptr) == CF_ERR_INVALID_ARG);
            c2 = codes; c2[3] = nullptr;
            EXPECT(cf_compress(ctx, 0, n, x.data(), recon.data(), err.data(), c2.data(), scales.data(), nullptr) == CF_ERR_INVALID_ARG);
            std::vector<void *> s2 = scales;
            s2[3] = nullptr;                                                    // the sparsifier has no scales: allowed
            EXPECT(cf_step_fused(ctx, 0, n, x.data(), recon.data(), err.data(), codes.data(), s2.data(), nullptr) == CF_OK);
            joined();
            EXPECT(cf_decompress(ctx, 0, n, (const void *const *)codes.data(), (const void *const *)recon.data(), recon.data(), nullptr) == CF_ERR_INVALID_ARG);
            EXPECT(joined().empty());
        }
        // launch sequences
        EXPECT(cf_step_fused(ctx, 0, n, x.data(), recon.data(), err.data(), codes.data(), scales.data(), nullptr) == CF_OK);
        EXPECT(uploaded(joined()));              // a pointer changed since the last call
        EXPECT(cf_step_fused(ctx, 0, n, x.data(), recon.data(), err.data(), codes.data(), scales.data(), nullptr) == CF_OK);
        std::string seq = joined();
        if (flags & CF_FLAG_TWO_KERNEL) EXPECT(seq.find("k_colreduce k_finalize k_encode k_encode_nm k_encode_nm k_lr_orth") != std::string::npos);
        if (flags & CF_FLAG_SINGLE_PASS) EXPECT(seq.find("k_reset_partials k_single_pass k_single_pass_redo k_encode k_encode_nm k_encode_nm k_lr_orth") != std::string::npos);
        if (flags & CF_FLAG_LOWRANK_INT4) EXPECT(seq.find("k_lr_quant_u") != std::string::npos);
        EXPECT(!uploaded(seq));                   // same pointers, same stream: no upload
        EXPECT(cf_step_fused(ctx, 2, 3, x.data() + 2, recon.data() + 2, err.data() + 2, codes.data() + 2, scales.data() + 2, nullptr) == CF_OK);
        seq = joined();
        EXPECT(seq.find("k_single_pass") == std::string::npos && seq.find("k_colreduce") == std::string::npos && seq.find("k_encode ") != std::string::npos);
        EXPECT(cf_step_fused(ctx, 0, 0, x.data(), recon.data(), err.data(), codes.data(), scales.data(), nullptr) == CF_OK && joined().empty());
        // another stream, then a captured call: the table is uploaded again each time, and once more afterwards
        EXPECT(cf_step_fused(ctx, 0, n, x.data(), recon.data(), err.data(), codes.data(), scales.data(), (void *)0x1000) == CF_OK);
        EXPECT(uploaded(joined()));
        g_capturing = true;
        EXPECT(cf_step_fused(ctx, 0, n, x.data(), recon.data(), err.data(), codes.data(), scales.data(), (void *)0x1000) == CF_OK);
        EXPECT(uploaded(joined()));
        g_capturing = false;
        EXPECT(cf_step_fused(ctx, 0, n, x.data(), recon.data(), err.data(), codes.data(), scales.data(), (void *)0x1000) == CF_OK);
        EXPECT(uploaded(joined()));
        EXPECT(cf_step_fused(ctx, 0, n, x.data(), recon.data(), err.data(), codes.data(), scales.data(), (void *)0x1000) == CF_OK);
        EXPECT(!uploaded(joined()));
        // receiver, profile hooks, bookkeeping calls
        EXPECT(cf_decompress(ctx, 0, n, (const void *const *)codes.data(), (const void *const *)scales.data(), recon.data(), (void *)0x1000) == CF_OK);
        seq = joined();
        EXPECT(seq.find("k_decode") != std::string::npos && seq.find("k_lr_apply") != std::string::npos);
        void *events[8] = {(void *)1, (void *)2, (void *)3, (void *)4, (void *)5, (void *)6, (void *)7, (void *)8};
        EXPECT(cf_profile_next_call(ctx, events, 4) == CF_OK);
        EXPECT(cf_compress(ctx, 0, 2, x.data(), (const void *const *)recon.data(), err.data(), codes.data(), scales.data(), (void *)0x1000) == CF_OK);
        EXPECT(cf_profile_launch_count(ctx) >= 2 && cf_profile_kernel_name(ctx, 0) != nullptr && cf_profile_kernel_name(ctx, 99) == nullptr);
        joined();
        uint32_t gave_up = 7;
        EXPECT(cf_given_up_items(ctx, nullptr, &gave_up) == CF_OK && gave_up == 0);
        EXPECT(cf_check_device(ctx, nullptr) == CF_OK && cf_last_hip_error(ctx) == 0);
        EXPECT(cf_set_warm(ctx, 0, n, 0) == CF_OK);
        EXPECT(cf_decompress(ctx, 0, n, (const void *const *)codes.data(), (const void *const *)scales.data(), recon.data(), nullptr) == CF_ERR_STATE);
        EXPECT(cf_set_warm(ctx, 0, n + 1, 1) == CF_ERR_INVALID_ARG);
        cf_destroy(ctx);
        for (auto *p : buf) delete p;
        std::free(ws);
    }
    cf_destroy(nullptr);

    // ---- which path a call takes by default: the single pass for tensors of 256 tokens and more in calls of 64
    // items and more, two kernels for tiny ones and for tensors so tall that more than 48 workgroups share a scale
    {
        struct Case { int64_t n, c; const char *must, *must_not; uint32_t flags; };
        const Case cases[] = {
            {4096, 512, "k_reset_partials k_single_pass k_single_pass_redo", "k_colreduce", 0},       // 16 items per group, 64 in all
            {16384, 64, "k_colreduce k_finalize k_encode", "k_single_pass", 0},                        // 64 items per group
            {16384, 64, "k_reset_partials k_single_pass k_single_pass_redo", "k_colreduce", CF_FLAG_SINGLE_PASS},
            {4096, 256, "k_colreduce k_finalize k_encode", "k_single_pass", 0},                        // 32 items in all: a tiny call
            {128, 8192, "k_colreduce k_finalize k_encode", "k_single_pass", 0},                        // a short tensor
            {4096, 512, "k_colreduce k_finalize k_encode", "k_single_pass", CF_FLAG_TWO_KERNEL},
        };
        for (const Case &cs : cases) {
            std::memset(&o, 0, sizeof o);
            o.flags = cs.flags;
            cf_tensor_desc d = desc(cs.n, cs.c, CF_BF16, 2, CF_SCALE_CHANNEL);
            Buffers b(d, &o);
            const size_t wsb = cf_workspace_bytes(&d, 1, &o);
            void *ws = nullptr;
            if (posix_memalign(&ws, 256, wsb) != 0) std::abort();
            cf_ctx *ctx = nullptr;
            EXPECT(cf_init(&ctx, &d, 1, &o, ws, wsb, nullptr) == CF_OK);
            const void *x = b.x;
            EXPECT(cf_warmup(ctx, 0, 1, &x, &b.recon, &b.err, nullptr) == CF_OK);
            joined();
            EXPECT(cf_step_fused(ctx, 0, 1, &x, &b.recon, &b.err, &b.codes, &b.scales, nullptr) == CF_OK);
            const std::string seq = joined();
            EXPECT(seq.find(cs.must) != std::string::npos);
            EXPECT(seq.find(cs.must_not) == std::string::npos);
            // new pointers (codes, scales) since the warm-up: a single pass takes them along in its first kernel
            if (std::string(cs.must).find("k_single_pass") != std::string::npos)
                EXPECT(seq.find("ptrs_in_reset k_reset_partials") != std::string::npos && seq.find("k_upload_ptrs") == std::string::npos);
            else
                EXPECT(seq.find("k_upload_ptrs") != std::string::npos && seq.find("ptrs_in_reset") == std::string::npos);
            cf_destroy(ctx);
            std::free(ws);
        }
    }

    // ---- the entry point that brings no workspace
    {
        std::memset(&o, 0, sizeof o);
        std::vector<cf_tensor_desc> many(40, desc(4096, 3072, CF_BF16, 2, CF_SCALE_CHANNEL));
        const void *nothing[40] = {};
        EXPECT(cf_step_fused_static(many.data(), 40, &o, nothing, (void *const *)nothing, (void *const *)nothing, (void *const *)nothing,
                                    (void *const *)nothing, nullptr) == CF_ERR_WORKSPACE);
        EXPECT(cf_workspace_bytes(many.data(), 40, &o) > CF_STATIC_SCRATCH_BYTES);
        for (int round = 0; round < 3; ++round) {
            std::vector<cf_tensor_desc> some = round == 1 ? std::vector<cf_tensor_desc>{desc(256, 64, CF_F32, 2, CF_SCALE_CHANNEL)}
                                                          : std::vector<cf_tensor_desc>{desc(2048, 1024, CF_BF16, 1, CF_SCALE_CHANNEL), desc(300, 384, CF_BF16, 4, CF_SCALE_GROUP)};
            std::vector<Buffers *> buf;
            std::vector<const void *> x;
            std::vector<void *> recon, err, codes, scales;
            for (auto &d : some) {
                buf.push_back(new Buffers(d, &o));
                x.push_back(buf.back()->x); recon.push_back(buf.back()->recon); err.push_back(buf.back()->err);
                codes.push_back(buf.back()->codes); scales.push_back(buf.back()->scales);
            }
            EXPECT(cf_step_fused_static(some.data(), (int)some.size(), &o, x.data(), recon.data(), err.data(), codes.data(), scales.data(), nullptr) == CF_OK);
            EXPECT(!joined().empty());
            EXPECT(cf_step_fused_static(some.data(), (int)some.size(), &o, nullptr, recon.data(), err.data(), codes.data(), scales.data(), nullptr) == CF_ERR_INVALID_ARG);
            for (auto *p : buf) delete p;
        }
    }
    if (g_failed) { std::printf("%d expectations failed\n", g_failed); return 1; }
    std::printf("host half of the C ABI: all expectations hold\n");
    return 0;
}
