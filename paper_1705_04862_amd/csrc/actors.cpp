// Worker pool and synthetic environment of the parallel framework (host only, no GPU code).
// n_w persistent threads each own a contiguous range of the n_e environments and step them one
// after the other when the master publishes a new generation (Section 3, the workers' step of
// Algorithm 1: all actions of a timestep are applied by the n_w workers side by side).
#include "../../include/paac_actors.h"

#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstring>
#include <mutex>
#include <thread>
#include <vector>

namespace {

constexpr int kH = 84, kW = 84, kFrames = 4, kFrame = kH * kW, kObs = kFrames * kFrame;

// splitmix64 finaliser: a counter-based hash, so results do not depend on who computes them
inline uint64_t mix(uint64_t x) {
    x += 0x9e3779b97f4a7c15ull;
    x = (x ^ (x >> 30)) * 0xbf58476d1ce4e5b9ull;
    x = (x ^ (x >> 27)) * 0x94d049bb133111ebull;
    return x ^ (x >> 31);
}
inline uint64_t key(uint64_t seed, uint64_t env, uint64_t episode, uint64_t step, uint64_t what) {
    return mix(mix(mix(mix(seed ^ 0x5041414300000000ull) + env) + episode) + step * 64 + what);
}

struct Env { uint64_t episode = 0, step = 0; };

}  // namespace

struct paac_actors {
    int n_e = 0, n_w = 0, sprites = 0;
    uint64_t seed = 0;
    float p_done = 0.f;
    std::vector<Env> env;
    std::vector<std::thread> workers;
    std::mutex m;
    std::condition_variable cv_go, cv_done;
    // a step is a few microseconds of work per environment, so both sides first poll these for a
    // short while and only then sleep on the condition variables (a wake-up costs tens of us)
    std::atomic<uint64_t> generation{0};
    std::atomic<int> pending{0};
    std::atomic<bool> quit{false};
    static constexpr int kSpin = 4000;
    // arguments of the step in flight
    const int32_t* actions = nullptr;
    uint8_t* states = nullptr;
    float* rewards = nullptr;
    uint8_t* dones = nullptr;
    double last_seconds = 0.0;

    void render(uint8_t* frame, int e, const Env& s, int action) const {
        memset(frame, 0, kFrame);
        for (int k = 0; k < sprites; ++k) {
            const uint64_t h = key(seed, e, s.episode, s.step, 8 + k);
            // the action shifts the sprite: the observation is a function of what the agent did
            // unsigned throughout: any int action (negative ones included) lands inside the row
            const int x = (int)(((unsigned)(h & 0xffff) + 3u * (unsigned)action * (unsigned)(k + 1)) % (unsigned)(kW - 8));
            const int y = (int)((h >> 16) & 0xffff) % (kH - 8);
            const uint8_t v = (uint8_t)(64 + ((h >> 32) % 192));
            for (int dy = 0; dy < 8; ++dy) memset(frame + (y + dy) * kW + x, v, 8);
        }
    }
    void reset_one(int e, uint8_t* obs) {
        Env& s = env[e];
        s.step = 0;
        memset(obs, 0, kObs - kFrame);
        render(obs + (kFrames - 1) * kFrame, e, s, 0);
    }
    void step_one(int e) {
        Env& s = env[e];
        uint8_t* obs = states + (size_t)e * kObs;
        const int a = actions[e];
        const uint64_t hr = key(seed, e, s.episode, s.step, 1) % 100;
        rewards[e] = hr < 5 ? -1.f : (hr >= 95 ? 1.f : 0.f);
        const double u = (double)(key(seed, e, s.episode, s.step, 2) >> 11) * (1.0 / 9007199254740992.0);
        const bool done = u < (double)p_done;
        dones[e] = done ? 1 : 0;
        if (done) {
            ++s.episode;
            reset_one(e, obs);
        } else {
            ++s.step;
            memmove(obs, obs + kFrame, kObs - kFrame);
            render(obs + (kFrames - 1) * kFrame, e, s, a);
        }
    }
    void worker(int w) {
        const int e0 = (int)((long)w * n_e / n_w), e1 = (int)((long)(w + 1) * n_e / n_w);
        uint64_t seen = 0;
        for (;;) {
            bool go = false;
            for (int i = 0; i < kSpin && !go; ++i) {
                go = quit.load(std::memory_order_acquire) || generation.load(std::memory_order_acquire) != seen;
                if (!go) __builtin_ia32_pause();
            }
            if (!go) {
                std::unique_lock<std::mutex> lk(m);
                cv_go.wait(lk, [&] { return quit.load() || generation.load() != seen; });
            }
            if (quit.load(std::memory_order_acquire)) return;
            seen = generation.load(std::memory_order_acquire);
            for (int e = e0; e < e1; ++e) step_one(e);
            if (pending.fetch_sub(1, std::memory_order_acq_rel) == 1) {
                std::lock_guard<std::mutex> lk(m);      // pairs with the master's predicate check
                cv_done.notify_one();
            }
        }
    }
};

extern "C" {

int paac_actors_create(int32_t n_e, int32_t n_w, uint64_t seed, float p_done, int32_t sprites, paac_actors** out) {
    if (!out) return -1;
    *out = nullptr;
    if (n_e < 1 || n_w < 1 || n_w > n_e || !(p_done >= 0.f && p_done <= 1.f) || sprites < 0 || sprites > 4096) return -2;
    paac_actors* a = new paac_actors();
    a->n_e = n_e; a->n_w = n_w; a->seed = seed; a->p_done = p_done; a->sprites = sprites;
    a->env.resize(n_e);
    for (int w = 0; w < n_w; ++w) a->workers.emplace_back([a, w] { a->worker(w); });
    *out = a;
    return 0;
}

void paac_actors_destroy(paac_actors* a) {
    if (!a) return;
    {
        std::lock_guard<std::mutex> lk(a->m);
        a->quit.store(true, std::memory_order_release);
    }
    a->cv_go.notify_all();
    for (auto& t : a->workers) t.join();
    delete a;
}

int paac_actors_reset(paac_actors* a, uint8_t* states_host) {
    if (!a || !states_host) return -1;
    for (int e = 0; e < a->n_e; ++e) {
        a->env[e].episode = 0;
        a->reset_one(e, states_host + (size_t)e * kObs);
    }
    return 0;
}

int paac_actors_step(paac_actors* a, const int32_t* actions_host, uint8_t* states_host, float* rewards_host,
                     uint8_t* dones_host) {
    if (!a || !actions_host || !states_host || !rewards_host || !dones_host) return -1;
    const auto t0 = std::chrono::steady_clock::now();
    a->actions = actions_host; a->states = states_host; a->rewards = rewards_host; a->dones = dones_host;
    a->pending.store(a->n_w, std::memory_order_release);
    {
        std::lock_guard<std::mutex> lk(a->m);           // a worker about to sleep sees the new generation
        a->generation.fetch_add(1, std::memory_order_acq_rel);
    }
    a->cv_go.notify_all();
    bool done = false;
    for (int i = 0; i < paac_actors::kSpin && !done; ++i) {
        done = a->pending.load(std::memory_order_acquire) == 0;
        if (!done) __builtin_ia32_pause();
    }
    if (!done) {
        std::unique_lock<std::mutex> lk(a->m);
        a->cv_done.wait(lk, [&] { return a->pending.load(std::memory_order_acquire) == 0; });
    }
    a->last_seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    return 0;
}

double paac_actors_last_step_seconds(const paac_actors* a) { return a ? a->last_seconds : 0.0; }

}  // extern "C"
