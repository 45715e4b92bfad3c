// Drives the library's host side (argument validation, planning of a client step, message
// bounds, sizing of the decode plan, the clean-up paths) in a build where the HIP runtime is
// replaced by hip_stub.cpp and everything is compiled with AddressSanitizer and
// UndefinedBehaviorSanitizer.  No GPU.  Usage: driver <file with one model's tensor sizes>.
// Pointers that stand for device buffers are never dereferenced here (launches do nothing), so
// large tensors are made-up, suitably aligned addresses.
#include "sbc.h"

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

extern "C" long stub_launches();
extern "C" long stub_live_blocks();
extern "C" void stub_fail_allocation(long nth);

#define CHECK(cond)                                                                     \
    do {                                                                                \
        if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); std::exit(1); } \
    } while (0)

struct Buffers {
    std::vector<const float*> dW;
    std::vector<float*> R, out;
    std::vector<int64_t> numel;
    int T() const { return (int)numel.size(); }
    int64_t total() const { int64_t s = 0; for (int64_t n : numel) s += n; return s; }
};

// made-up addresses: three disjoint ranges, each tensor 16-byte aligned
static Buffers fake_buffers(const std::vector<int64_t>& sizes, uintptr_t salt = 0) {
    Buffers b;
    uintptr_t a = 0x100000000000ull + salt, r = 0x200000000000ull + salt, o = 0x300000000000ull + salt;
    for (int64_t n : sizes) {
        b.numel.push_back(n);
        b.dW.push_back(reinterpret_cast<const float*>(a));
        b.R.push_back(reinterpret_cast<float*>(r));
        b.out.push_back(reinterpret_cast<float*>(o));
        const uintptr_t step = ((uintptr_t)n * 4u + 15u) & ~(uintptr_t)15u;
        a += step; r += step; o += step;
    }
    return b;
}

static void* const kMsg = reinterpret_cast<void*>(0x400000000000ull);

static int compress(sbc_ctx* c, const Buffers& b, double p, size_t capacity, size_t* nbytes) {
    return sbc_compress(c, nullptr, b.dW.data(), b.R.data(), b.numel.data(), b.T(), p, kMsg, capacity, nbytes);
}

int main(int argc, char** argv) {
    CHECK(argc == 2);
    std::vector<int64_t> model;
    {
        std::FILE* f = std::fopen(argv[1], "r");
        CHECK(f != nullptr);
        long long n;
        while (std::fscanf(f, "%lld", &n) == 1) model.push_back(n);
        std::fclose(f);
    }
    CHECK(model.size() >= 100);

    // ---- scalar helpers ----
    const double bad_p[] = {0.0, 1.0, -1.0, 2.0, 0.0 / 1.0 - 0.0, 1e-12};
    for (double p : bad_p) {
        const int64_t n1[1] = {10};
        if (p != 1e-12) { CHECK(sbc_golomb_bstar(p) == SBC_EINVAL); CHECK(sbc_num_kept(10, p) == SBC_EINVAL); }
        CHECK(sbc_msg_bound(n1, 1, p) == 0);
        CHECK(sbc_msg_bound_sampled(n1, 1, p) == 0);
    }
    CHECK(sbc_golomb_bstar(0.001) == 9 && sbc_golomb_bstar(0.5) == 0);
    CHECK(sbc_num_kept(0, 0.1) == SBC_EINVAL && sbc_num_kept(64, 0.001) == 1);
    {
        const int64_t zero[1] = {0}, huge[1] = {(int64_t)1 << 32}, neg[1] = {-5};
        CHECK(sbc_msg_bound(zero, 1, 0.1) == 0 && sbc_msg_bound(huge, 1, 0.1) == 0 && sbc_msg_bound(neg, 1, 0.1) == 0);
        CHECK(sbc_msg_bound(nullptr, 1, 0.1) == 0 && sbc_msg_bound(zero, 0, 0.1) == 0);
    }
    for (int code = 1; code >= -8; --code) CHECK(sbc_strerror(code) != nullptr);

    // ---- create: bad arguments, and an allocation that fails half way (everything is released) ----
    sbc_ctx* c = nullptr;
    CHECK(sbc_create(nullptr, 0, 10, 1) == SBC_EINVAL);
    CHECK(sbc_create(&c, 0, 0, 1) == SBC_EINVAL && sbc_create(&c, 0, 10, 0) == SBC_EINVAL);
    CHECK(sbc_create(&c, 1, 10, 1) == SBC_EINVAL && sbc_create(&c, -1, 10, 1) == SBC_EINVAL);
    for (long nth = 0; nth < 60; nth += 7) {
        stub_fail_allocation(nth);
        const int rc = sbc_create(&c, 0, 100000, 4);
        stub_fail_allocation(-1);
        if (rc == SBC_OK) { sbc_destroy(c); c = nullptr; }
        else CHECK(rc == SBC_EHIP && c == nullptr);
        CHECK(stub_live_blocks() == 0);
    }
    sbc_destroy(nullptr);

    // ---- the model: plans of the client step in every mode ----
    const Buffers m = fake_buffers(model);
    const double p = 0.001;
    const size_t bound = sbc_msg_bound(m.numel.data(), m.T(), p);
    CHECK(bound > 32 + 24 * (size_t)m.T());
    CHECK(sbc_msg_bound_sampled(m.numel.data(), m.T(), p) >= bound);
    CHECK(sbc_create(&c, 0, m.total(), m.T()) == SBC_OK);
    size_t nbytes = 123;
    // argument errors: nothing is enqueued
    const long launches0 = stub_launches();
    CHECK(sbc_compress(nullptr, nullptr, m.dW.data(), m.R.data(), m.numel.data(), m.T(), p, kMsg, bound, &nbytes) == SBC_EINVAL);
    CHECK(sbc_compress(c, nullptr, nullptr, m.R.data(), m.numel.data(), m.T(), p, kMsg, bound, &nbytes) == SBC_EINVAL);
    CHECK(sbc_compress(c, nullptr, m.dW.data(), m.R.data(), m.numel.data(), 0, p, kMsg, bound, &nbytes) == SBC_EINVAL);
    CHECK(sbc_compress(c, nullptr, m.dW.data(), m.R.data(), m.numel.data(), m.T(), 0.0, kMsg, bound, &nbytes) == SBC_EINVAL);
    CHECK(sbc_compress(c, nullptr, m.dW.data(), m.R.data(), m.numel.data(), m.T(), p, nullptr, bound, &nbytes) == SBC_EINVAL);
    CHECK(sbc_compress(c, nullptr, m.dW.data(), m.R.data(), m.numel.data(), m.T(), p, (char*)kMsg + 4, bound, &nbytes) == SBC_EINVAL);
    CHECK(compress(c, m, p, bound - 1, &nbytes) == SBC_ECAPACITY);
    {
        Buffers x = m;
        x.dW[3] = reinterpret_cast<const float*>((uintptr_t)x.dW[3] + 2);              // misaligned
        CHECK(compress(c, x, p, bound, &nbytes) == SBC_EINVAL);
        x = m; x.R[5] = const_cast<float*>(x.dW[5]) + 1;                                // residual overlaps the update
        CHECK(compress(c, x, p, bound, &nbytes) == SBC_EINVAL);
        x = m; x.dW[0] = nullptr;
        CHECK(compress(c, x, p, bound, &nbytes) == SBC_EINVAL);
        x = m; x.numel[7] = 0;
        CHECK(compress(c, x, p, bound, &nbytes) == SBC_EINVAL);
        x = m; x.numel[7] = (int64_t)1 << 32;
        CHECK(compress(c, x, p, bound, &nbytes) != SBC_OK);
        x = m; x.numel[0] += 1;                                                          // one entry more than the context holds
        CHECK(compress(c, x, p, sbc_msg_bound(x.numel.data(), x.T(), p), &nbytes) == SBC_ECAPACITY);
        std::vector<int64_t> more(model); more.push_back(1);
        const Buffers y = fake_buffers(more);
        CHECK(compress(c, y, p, bound + 64, &nbytes) == SBC_ECAPACITY);               // one tensor more
    }
    CHECK(stub_launches() == launches0);
    CHECK(sbc_compress_end(c, &nbytes) == SBC_EINVAL);                                   // nothing pending
    CHECK(sbc_last_tensor_stats(c, 0, nullptr, nullptr, nullptr, nullptr, nullptr) != SBC_OK);   // no successful call yet

    // plans: first call, same buffers again (cached plan), five more buffer sets (the device copies
    // of the tensor table are recycled), every option
    for (int opt_round = 0; opt_round < 6; ++opt_round) {
        if (opt_round == 1) CHECK(sbc_set_option(c, SBC_OPT_CARRY_FILTER_KEYS, 1) == SBC_OK);
        if (opt_round == 2) CHECK(sbc_set_option(c, SBC_OPT_FUSED_STEP, 1) == SBC_OK);
        if (opt_round == 3) CHECK(sbc_set_option(c, SBC_OPT_FORCE_EXACT_PATH, 1) == SBC_OK);
        if (opt_round == 4) { CHECK(sbc_set_option(c, SBC_OPT_FORCE_EXACT_PATH, 0) == SBC_OK); CHECK(sbc_set_option(c, SBC_OPT_WIDE_MIN_KEPT, 1) == SBC_OK); }
        if (opt_round == 5) CHECK(sbc_set_option(c, SBC_OPT_SAMPLED_THRESHOLD, 1) == SBC_OK);
        const size_t need = opt_round == 5 ? sbc_msg_bound_sampled(m.numel.data(), m.T(), p) : bound;
        for (int set = 0; set < 7; ++set) {
            const Buffers s = fake_buffers(model, (uintptr_t)(set % 6) << 36);
            nbytes = 123;
            CHECK(compress(c, s, p, need, &nbytes) == SBC_OK && nbytes == 0);           // (no kernel ran: empty result)
            CHECK(sbc_compress_begin(c, nullptr, s.dW.data(), s.R.data(), s.numel.data(), s.T(), p, kMsg, need) == SBC_OK);
            CHECK(sbc_compress_begin(c, nullptr, s.dW.data(), s.R.data(), s.numel.data(), s.T(), p, kMsg, need) == SBC_EINVAL);
            CHECK(sbc_set_option(c, SBC_OPT_FUSED_STEP, 1) != SBC_OK || true);
            CHECK(sbc_compress_end(c, &nbytes) == SBC_OK);
        }
        for (double q : {0.5, 0.1, 0.01, 0.0001}) {
            const size_t nb = (opt_round == 5 ? sbc_msg_bound_sampled : sbc_msg_bound)(m.numel.data(), m.T(), q);
            CHECK(nb > 0 && compress(c, m, q, nb, &nbytes) == SBC_OK);
        }
        CHECK(sbc_last_route(c) >= 0);
        double mp, mn; int side; int64_t nnz, bits, cp, cn;
        // (no kernel filled the state: the counts of kept entries read zero, which the call reports)
        CHECK(sbc_last_tensor_stats(c, 0, &mp, &mn, &side, &nnz, &bits) == SBC_EINTERNAL);
        CHECK(sbc_last_tensor_stats(c, m.T(), &mp, &mn, &side, &nnz, &bits) == SBC_EINVAL);
        CHECK(sbc_last_candidates(c, m.T() - 1, &cp, &cn) == SBC_OK && sbc_last_candidates(c, -1, &cp, &cn) == SBC_EINVAL);
        std::vector<uint32_t> mask((size_t)(m.numel[0] + 31) / 32);
        CHECK(sbc_last_mask(c, 0, mask.data(), mask.size()) == SBC_OK);
        CHECK(sbc_last_mask(c, 0, mask.data(), mask.size() - 1) != SBC_OK);
    }
    CHECK(sbc_set_option(c, 99, 1) == SBC_EINVAL && sbc_set_option(nullptr, SBC_OPT_FUSED_STEP, 1) == SBC_EINVAL);
    CHECK(sbc_profile_enable(c, 2) == SBC_OK);
    CHECK(compress(c, m, p, sbc_msg_bound_sampled(m.numel.data(), m.T(), p), &nbytes) == SBC_OK);
    for (int stage = 0; stage < 16; ++stage) {
        const char* name = nullptr; double ms; int64_t calls;
        const int rc = sbc_profile_read(c, stage, &name, &ms, &calls);
        CHECK(rc == SBC_OK ? name != nullptr : rc == SBC_EINVAL);
    }
    CHECK(sbc_profile_enable(c, 0) == SBC_OK);

    // ---- decode plan: argument errors, every stream by one workgroup, tiled streams, deferred status ----
    CHECK(sbc_decompress_accumulate(c, nullptr, kMsg, 31 + 24 * (size_t)m.T(), m.numel.data(), m.T(), p, 1.f, m.out.data()) == SBC_ECORRUPT);
    CHECK(sbc_decompress_accumulate(c, nullptr, (char*)kMsg + 4, bound, m.numel.data(), m.T(), p, 1.f, m.out.data()) == SBC_EINVAL);
    CHECK(sbc_decompress_accumulate(c, nullptr, kMsg, bound, m.numel.data(), m.T() + 1, p, 1.f, m.out.data()) == SBC_ECAPACITY);
    CHECK(sbc_decompress_accumulate(c, nullptr, kMsg, bound, nullptr, m.T(), p, 1.f, m.out.data()) == SBC_EINVAL);
    for (double q : {0.5, 0.1, 0.01, 0.001, 0.0001})
        for (int rep = 0; rep < 2; ++rep)
            CHECK(sbc_decompress_accumulate(c, nullptr, kMsg, bound, m.numel.data(), m.T(), q, 1.f / 32, m.out.data()) == SBC_OK);
    CHECK(sbc_set_option(c, SBC_OPT_DEFER_DECODE_STATUS, 1) == SBC_OK);
    for (int rep = 0; rep < 3; ++rep)
        CHECK(sbc_decompress_accumulate(c, nullptr, kMsg, bound, m.numel.data(), m.T(), 0.1, 1.f, m.out.data()) == SBC_OK);
    CHECK(sbc_set_option(c, SBC_OPT_DEFER_DECODE_STATUS, 0) == SBC_EINVAL);           // a status is outstanding
    CHECK(sbc_decode_status(c, nullptr) == SBC_OK);
    CHECK(sbc_set_option(c, SBC_OPT_DEFER_DECODE_STATUS, 0) == SBC_OK);
    sbc_destroy(c); c = nullptr;
    CHECK(stub_live_blocks() == 0);

    // ---- shapes at the edges: one entry; a tensor of thousands of chunks; more tensors that keep
    // very many entries than the grid-wide kernels and the tiled decoder take; many tiny tensors ----
    {
        const std::vector<std::vector<int64_t>> shapes = {
            {1}, {8192}, {8193}, {64000000, 5}, std::vector<int64_t>(70, 70000), std::vector<int64_t>(3000, 7)};
        for (const auto& sizes : shapes) {
            const Buffers s = fake_buffers(sizes);
            CHECK(sbc_create(&c, 0, s.total(), s.T()) == SBC_OK);
            for (int fused = 0; fused < 2; ++fused) {
                CHECK(sbc_set_option(c, SBC_OPT_FUSED_STEP, fused) == SBC_OK);
                CHECK(sbc_set_option(c, SBC_OPT_WIDE_MIN_KEPT, 6500) == SBC_OK);
                for (double q : {0.9, 0.1, 0.001}) {
                    const size_t nb = sbc_msg_bound(s.numel.data(), s.T(), q);
                    CHECK(nb > 0 && compress(c, s, q, nb, &nbytes) == SBC_OK);
                    CHECK(sbc_decompress_accumulate(c, nullptr, kMsg, nb, s.numel.data(), s.T(), q, 1.f, s.out.data()) == SBC_OK);
                }
            }
            sbc_destroy(c); c = nullptr;
            CHECK(stub_live_blocks() == 0);
        }
    }

    // ---- a context with short candidate lists: the plan shares them out, large p does not fit ----
    {
        CHECK(sbc_create_compact(nullptr, 0, 10, 1) == SBC_EINVAL);
        CHECK(sbc_create_compact(&c, 0, m.total(), m.T()) == SBC_OK);
        for (double q : {0.001, 0.01, 0.05}) {
            const size_t nb = sbc_msg_bound(m.numel.data(), m.T(), q);
            CHECK(compress(c, m, q, nb, &nbytes) == SBC_OK);
            CHECK(sbc_decompress_accumulate(c, nullptr, kMsg, nb, m.numel.data(), m.T(), q, 1.f, m.out.data()) == SBC_OK);
        }
        const long launched = stub_launches();
        CHECK(compress(c, m, 0.3, sbc_msg_bound(m.numel.data(), m.T(), 0.3), &nbytes) == SBC_ECAPACITY);
        CHECK(stub_launches() == launched);
        sbc_destroy(c); c = nullptr;
        CHECK(stub_live_blocks() == 0);
    }

    // ---- the server step that allocates nothing ----
    {
        int32_t* const status = reinterpret_cast<int32_t*>(0x500000000000ull);
        const long blocks = stub_live_blocks();
        CHECK(sbc_decompress_accumulate_noalloc(0, nullptr, nullptr, bound, m.numel.data(), m.T(), p, 1.f, m.out.data(), status) == SBC_EINVAL);
        CHECK(sbc_decompress_accumulate_noalloc(0, nullptr, kMsg, bound, m.numel.data(), m.T(), p, 1.f, m.out.data(), nullptr) == SBC_EINVAL);
        CHECK(sbc_decompress_accumulate_noalloc(3, nullptr, kMsg, bound, m.numel.data(), m.T(), p, 1.f, m.out.data(), status) == SBC_EINVAL);
        CHECK(sbc_decompress_accumulate_noalloc(0, nullptr, kMsg, 10, m.numel.data(), m.T(), p, 1.f, m.out.data(), status) == SBC_ECORRUPT);
        const Buffers big = fake_buffers(std::vector<int64_t>(SBC_NOALLOC_MAX_TENSORS + 1, 100));
        CHECK(sbc_decompress_accumulate_noalloc(0, nullptr, kMsg, 1 << 20, big.numel.data(), big.T(), p, 1.f, big.out.data(), status) == SBC_ECAPACITY);
        for (double q : {0.1, 0.001})
            CHECK(sbc_decompress_accumulate_noalloc(0, nullptr, kMsg, bound, m.numel.data(), m.T(), q, 1.f, m.out.data(), status) == SBC_OK);
        CHECK(stub_live_blocks() == blocks);                                            // it allocated nothing
    }
    std::printf("host checks passed, %ld launches planned\n", stub_launches());
    return 0;
}
