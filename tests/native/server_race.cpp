// Host-only build of the serving front end (queues, scheduling and execution threads, policy, predictor, link model)
// driven by a fake executor from several client threads, for the race and memory sanitizers.  The GPU-side entry
// points the front end links against are stubbed: with an external executor it never calls them.
#include <atomic>
#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <map>
#include <mutex>
#include <thread>
#include <vector>
#include "strait.h"
namespace strait { void set_error(const char* fmt, ...) { (void)fmt; } const char* last_error() { return ""; } }
extern "C" {
// GPU-side entry points the server links against; never called with an external executor
strait_status strait_model_info(const strait_model*, int32_t*, int32_t*, int32_t*, int32_t*, int32_t*) { return -1; }
strait_status strait_model_io(const strait_model*, int32_t, size_t*, size_t*) { return -1; }
strait_status strait_model_layer(const strait_model*, int32_t, strait_layer_info*) { return -1; }
strait_status strait_model_staging(const strait_model*, int32_t, void**, size_t*) { return -1; }
strait_status strait_submit(strait_model*, strait_priority, int32_t, const void*, const int32_t*, void*, strait_ticket*) { return -1; }
strait_status strait_wait(strait_ticket, strait_record*) { return -1; }
}
struct Fake { std::mutex mu; std::map<uint64_t, std::chrono::steady_clock::time_point> start; std::atomic<int> live{0}; };
static int32_t f_submit(void* u, uint64_t seq, int32_t, int32_t, int32_t, const void* const*, void* const*, const int32_t*) {
    Fake* f = (Fake*)u; std::lock_guard<std::mutex> lk(f->mu); f->start[seq] = std::chrono::steady_clock::now(); f->live++; return 0; }
static int32_t f_wait(void* u, uint64_t seq, double* k, double* h) {
    Fake* f = (Fake*)u; std::chrono::steady_clock::time_point t0;
    { std::lock_guard<std::mutex> lk(f->mu); t0 = f->start[seq]; }
    std::this_thread::sleep_until(t0 + std::chrono::microseconds(800));
    f->live--; *k = 600000.0; *h = 10000.0; return 0; }
int main() {
    strait_sched* sc = nullptr; strait_sched_create(1, nullptr, &sc);
    strait_batch_profile prof[8];
    for (int b = 0; b < 8; ++b) { prof[b] = strait_batch_profile{}; prof[b].t_inf_isol_ns = 8e5 + 1e4 * b; prof[b].t_htod_ns = 10000; prof[b].t_kernel_isol_ns = 6e5; for (int i = 0; i < 5; ++i) prof[b].m[i] = 0.05; prof[b].m_self_cmp = prof[b].m_self_mem = 0.05; }
    strait_sched_set_profile(sc, 1, 0, prof, 8); strait_sched_set_profile(sc, 2, 1, prof, 8);
    Fake fk; strait_executor ex{&fk, f_submit, f_wait};
    strait_server* sv = nullptr; strait_server_create(sc, 4, 200000, &ex, &sv);
    strait_server_model m1{nullptr, 1, 0, 8, 3, 20000000, 300000}, m2{nullptr, 2, 1, 8, 3, 50000000, 1000000};
    strait_server_add_model(sv, &m1); strait_server_add_model(sv, &m2);
    strait_server_start(sv);
    std::vector<std::thread> th;
    std::atomic<long> sent{0};
    for (int t = 0; t < 6; ++t) th.emplace_back([&, t] { for (int i = 0; i < 2000; ++i) { uint64_t id; if (strait_server_request(sv, 1 + (t + i) % 2, nullptr, 0, nullptr, &id) == 0) sent++; if (i % 7 == 0) std::this_thread::sleep_for(std::chrono::microseconds(50)); } });
    std::thread poll([&] { strait_request_record r[256]; strait_server_stats st; for (int i = 0; i < 400; ++i) { int32_t n; strait_server_results(sv, r, 256, &n); strait_server_get_stats(sv, &st); std::this_thread::sleep_for(std::chrono::milliseconds(1)); } });
    for (auto& x : th) x.join();
    int rc = strait_server_wait_idle(sv, 20000000000LL);
    poll.join();
    strait_server_stats st; strait_server_get_stats(sv, &st);
    printf("sent %ld idle rc %d requests %lld served %lld dropped %lld batches %lld max in flight %lld\n", sent.load(), rc, (long long)st.requests, (long long)st.served, (long long)st.dropped, (long long)st.batches, (long long)st.max_in_flight);
    // stop with work in flight
    for (int i = 0; i < 50; ++i) strait_server_request(sv, 1, nullptr, 0, nullptr, nullptr);
    strait_server_stop(sv); strait_server_destroy(sv); strait_sched_destroy(sc);
    return st.requests == sent.load() && st.served + st.dropped == st.requests ? 0 : 1;
}
