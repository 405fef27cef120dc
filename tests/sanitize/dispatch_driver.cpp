// Drives the host-side dispatching code (one translation unit with it) under AddressSanitizer /
// UndefinedBehaviorSanitizer: random pushes and pops on buffers of several shapes (full and empty included), controller
// observations, and dispatcher loops that overflow the storage.  Prints a checksum; any sanitizer report aborts the run.
#include "../../paper_2408_12526_amd/csrc/sp_dispatch.cpp"

#include <cstdio>

static unsigned long long lcg = 1234567ULL;
static unsigned rnd(unsigned n)
{
    lcg = lcg * 6364136223846793005ULL + 1442695040888963407ULL;
    return (unsigned)((lcg >> 33) % n);
}

int main()
{
    long long sum = 0;
    const int shapes[4][4] = {{8, 128, 4, 4}, {8, 128, 4, 64}, {16, 96, 1, 3}, {1, 7, 3, 1000}};
    for (auto& sh : shapes) {
        sp_lab* b = nullptr;
        if (sp_lab_create(sh[0], sh[1], sh[2], sh[3], &b) != SP_OK) return 2;
        std::vector<int64_t> ids((size_t)sh[2]);
        std::vector<int32_t> lens((size_t)sh[2]);
        for (int op = 0; op < 20000; ++op) {
            if (rnd(3)) {
                int32_t joined = 0;
                const int rc = sp_lab_push(b, op, (int32_t)rnd(300) - 20, &joined);
                if (rc != SP_OK && rc != SP_EFULL) return 3;
                sum += joined + rc;
            } else {
                int32_t bin, bl, cnt;
                const int rc = sp_lab_pop(b, &bin, &bl, ids.data(), lens.data(), &cnt);
                if (rc != SP_OK && rc != SP_EEMPTY) return 4;
                if (rc == SP_OK) sum += bin + bl + cnt + ids[(size_t)cnt - 1] + lens[0];
            }
            sum += sp_lab_elements(b) + sp_lab_samples(b) + sp_lab_bin_of(b, (int32_t)rnd(400)) + sp_lab_bin_len(b, 0);
        }
        sp_lab_free(b);
    }
    sp_lab* none = nullptr;
    if (sp_lab_create(0, 128, 4, 4, &none) == SP_OK || sp_lab_create(8, 128, 4, 0, &none) == SP_OK) return 5;
    sp_ctl* ctl = nullptr;
    if (sp_ctl_create(8, 8, 1, 1000, 8, &ctl) != SP_OK) return 6;
    for (int i = 0; i < 5000; ++i) {
        sum += rnd(2) ? sp_ctl_on_buffered(ctl, (int32_t)rnd(10)) : sp_ctl_on_tick(ctl, i * 37, (int32_t)rnd(3), (int32_t)rnd(9));
        sum += sp_ctl_k(ctl) + sp_ctl_groups(ctl);
    }
    sp_ctl_free(ctl);
    const int64_t n = 4000;
    std::vector<int64_t> arr((size_t)n), disp((size_t)n), done((size_t)n), elem((size_t)n), etok((size_t)n), tus(64);
    std::vector<int32_t> len((size_t)n), kused((size_t)n), esize((size_t)n), tk(64);
    int64_t t = 0;
    for (int64_t i = 0; i < n; ++i) { t += rnd(40); arr[(size_t)i] = t; len[(size_t)i] = (int32_t)rnd(200) + 1; }
    const int64_t base[9] = {0, 100, 110, 120, 130, 140, 150, 160, 170}, per[9] = {0, 200, 220, 240, 260, 280, 300, 320, 340};
    for (int padded = 0; padded < 2; ++padded)
        for (int cap : {2, 64, 4096}) {
            sp_sim_config cfg{};
            cfg.total_students = 8; cfg.slots = 8; cfg.k_min = padded ? 8 : 1; cfg.k_start = 8; cfg.window_us = 500;
            cfg.bin_width = 8; cfg.max_len = 128; cfg.max_elem = 4; cfg.capacity = cap; cfg.padded = padded;
            cfg.base_us = base; cfg.per_token_ns = per;
            int64_t ne = 0, nt = 0, ref = 0;
            const int rc = sp_dispatch_simulate(&cfg, arr.data(), len.data(), n, disp.data(), done.data(), kused.data(),
                                                elem.data(), etok.data(), esize.data(), &ne, tus.data(), tk.data(), 64, &nt,
                                                &ref);
            if (rc != SP_OK) return 7;
            sum += ne + nt + ref + done[(size_t)n - 1];
        }
    std::printf("dispatch driver checksum %lld\n", sum);
    return 0;
}
