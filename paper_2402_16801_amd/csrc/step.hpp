// One Craftax-Classic step of one environment, executed by the G lanes that own it.
//
// What the paper fixes: 17 actions that are always legal and fall back to a no-op when their
// prerequisites are missing (section "RL Environment Interface"), 22 achievements worth +1
// the first time and +-0.1 per health point (same section), fixed-capacity creature and plant
// tables whose empty slots are masked (appendix "Differences between Craftax-Classic and
// Crafter"), creature health and damage (appendix "Creatures").  The remaining rules
// ("mimic Crafter") are this library's own frozen reading.
//
// Random draws have fixed slots in four Philox blocks per step: word s < 3 of block b holds the
// draws of mob and plant slot b + 4s (bits 0..15 decision, 16..18 movement choice, 19..26 the
// plant's "eaten" draw); word 3 of block b is misc[b]: spawn attempt of type b < 3 (two 10-bit
// picks for x and y, a 12-bit probability draw) and, for b = 3, the sapling draw.  A lane owns
// slots l, l + G, ... with G a multiple of four, so block l & 3 holds all its draws: one Philox
// block per lane and step.
//
// Memory round trips of a step: record -> 9x11 map window around the player (kept in LDS,
// patched with this step's edits, and reused for the observation) -> one terrain byte per
// moving mob and per spawn candidate.
#pragma once

#include "common.hpp"

namespace cx {

enum Intent : int { K_NONE = 0, K_MOVE = 1, K_MOVE_PATH = 2, K_ATTACK = 3, K_SHOOT = 4, K_FLY = 5 };

struct StepOut { bool done; float reward; int mvx, mvy, woff; uint32_t unlocked; };   // unlocked: achievement bits new after this step

// The part of the window a step can touch, in window rows and columns (inclusive): the 7 x 9 view
// around the player, widened by one row or column on the side the player may move to.  Nothing
// else of the window is read by the rules or the renderer, so nothing else is fetched: nine rows
// always straddle two map tiles (cache lines), seven or eight often do not.
struct WinRect { int r0, r1, c0, c1; };
__device__ inline WinRect full_window() { return WinRect{0, WIN_ROWS - 1, 0, WIN_COLS - 1}; }
__device__ inline WinRect window_for_action(int a)
{
    WinRect w{1, WIN_ROWS - 2, 1, WIN_COLS - 2};
    if (a == AC_LEFT) w.c0 = 0;
    if (a == AC_RIGHT) w.c1 = WIN_COLS - 1;
    if (a == AC_UP) w.r0 = 0;
    if (a == AC_DOWN) w.r1 = WIN_ROWS - 1;
    return w;
}
__device__ inline bool in_rect(const WinRect& w, int wr, int wc) { return wr >= w.r0 && wr <= w.r1 && wc >= w.c0 && wc <= w.c1; }

// Loads the map window around (px, py) into LDS with aligned dword loads: lane l takes dwords
// l, l+G, ... of the 36 (four per window row).  A dword never straddles a map tile, and the
// whole window lies in at most four tiles (cache lines).  Only the dwords that hold a cell of
// `need` are fetched; the others are left as they are.
template <int G>
__device__ __forceinline__ void load_window(int l, int px, int py, const uint8_t* __restrict__ map, uint32_t* win, const WinRect need)
{
    constexpr int NIT = (WIN_DWORDS + G - 1) / G;
    const int x0 = px - WIN_COLS / 2, xa = x0 & ~3, y0 = py - WIN_ROWS / 2, woff = x0 & 3;
    const int d0 = (woff + need.c0) >> 2, d1 = (woff + need.c1) >> 2;     // first and last dword of a row that is needed
    uint32_t v[NIT];
    bool inside[NIT], wanted[NIT];
    // all loads are issued unconditionally (cells outside the map, and dwords that are not needed,
    // read the player's own dword, whose cache line is fetched anyway), so they go out back to back
    // and are waited for once
    const int idle = map_index(px, py) & ~3;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int d = l + it * G;
        const int r = d >> 2, j = d & 3, x = xa + (j << 2), y = y0 + r;
        wanted[it] = d < WIN_DWORDS && r >= need.r0 && r <= need.r1 && j >= d0 && j <= d1;
        inside[it] = wanted[it] && (unsigned)y < (unsigned)MAPW && (unsigned)x < (unsigned)MAPW;
        v[it] = *reinterpret_cast<const uint32_t*>(map + (inside[it] ? map_index(x, y) : idle));
    }
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int d = l + it * G;
        if (wanted[it]) win[CX_IDX(d, WIN_DWORDS)] = inside[it] ? v[it] : 0x01010101u * (uint32_t)BK_OOB;
    }
}
template <int G>
__device__ __forceinline__ void load_window(int l, int px, int py, const uint8_t* __restrict__ map, uint32_t* win)
{
    load_window<G>(l, px, py, map, win, full_window());
}

// Mob and plant slots stay in their packed record form while the step runs: bit 0 alive,
// bits 1..12 the cell (x | y<<6), so "is this live slot on cell c" is one AND and one compare
// against key(c) = 1 | x<<1 | y<<7, a move is one bit-field insert and a kill is "= 0".
constexpr uint32_t KEY_MASK = 0x1FFFu;
__device__ inline uint32_t cell_key(int x, int y) { return 1u | ((uint32_t)x << 1) | ((uint32_t)y << 7); }
__device__ inline int mob_x(uint32_t w) { return (int)__builtin_amdgcn_ubfe(w, 1, 6); }
__device__ inline int mob_y(uint32_t w) { return (int)__builtin_amdgcn_ubfe(w, 7, 6); }
__device__ inline uint32_t mob_moved(uint32_t w, uint32_t key) { return (w & ~KEY_MASK) | key; }

// Small per-block-id tables of the DO action, packed into 64-bit constants (ids 0..10):
// item picked up (+1, 0 = none), pickaxe needed (0 none, 1 wood, 2 stone, 3 iron), achievement.
constexpr uint64_t DO_ITEM = (6ull << (4 * BK_GRASS)) | (2ull << (4 * BK_STONE)) | (1ull << (4 * BK_TREE)) |
                             (3ull << (4 * BK_COAL)) | (4ull << (4 * BK_IRON)) | (5ull << (4 * BK_DIAMOND));
constexpr uint64_t DO_GATE = (1ull << (2 * BK_STONE)) | (1ull << (2 * BK_COAL)) | (2ull << (2 * BK_IRON)) | (3ull << (2 * BK_DIAMOND));
constexpr uint64_t DO_ACH = ((uint64_t)ACH_COLLECT_SAPLING << (5 * BK_GRASS)) | ((uint64_t)ACH_COLLECT_STONE << (5 * BK_STONE)) |
                            ((uint64_t)ACH_COLLECT_WOOD << (5 * BK_TREE)) | ((uint64_t)ACH_COLLECT_COAL << (5 * BK_COAL)) |
                            ((uint64_t)ACH_COLLECT_IRON << (5 * BK_IRON)) | ((uint64_t)ACH_COLLECT_DIAMOND << (5 * BK_DIAMOND));
constexpr uint32_t MINED_MASK = (1u << BK_STONE) | (1u << BK_COAL) | (1u << BK_IRON) | (1u << BK_DIAMOND);  // leave a path
constexpr uint32_t MAKE_ACH = ACH_MAKE_WOOD_PICKAXE | (ACH_MAKE_STONE_PICKAXE << 5) | (ACH_MAKE_IRON_PICKAXE << 10) |
                              (ACH_MAKE_WOOD_SWORD << 15) | (ACH_MAKE_STONE_SWORD << 20) | (ACH_MAKE_IRON_SWORD << 25);

// e: the environment's LDS area (record already loaded).  Returns with the record in LDS
// updated (unless the episode ended) and the window patched with this step's map edits;
// (mvx, mvy) is how far the player moved, i.e. where the view sits inside the window.
// KEEP_WIN (kernels that keep an environment in LDS from step to step): the window is only loaded
// if the one in LDS was not loaded for the player's current position; every change the step makes
// to the map inside the window is patched into it, so a kept window equals a fresh one.
template <int G, bool KEEP_WIN = false>
__device__ __forceinline__ StepOut step_env(int l, uint32_t env, uint32_t* e, uint8_t* __restrict__ map,
                                   const Luts* __restrict__ luts, int action, const Params& p)
{
    using Gr = Grp<G>;
    constexpr int NSM = Gr::NS_MOB, NSP = Gr::NS_PLANT;
    uint32_t* rec = e + LDS_REC;
    uint8_t* win = reinterpret_cast<uint8_t*>(e + LDS_WIN);

    // ---- unpack -----------------------------------------------------------------------------
    const uint32_t w_pos = rec[RW_POS], w_vit = rec[RW_VIT], w_cnt = rec[RW_CNT];
    uint32_t w_inv = rec[RW_INV];    // six 4-bit counts, six tool flags from bit 24: stays packed
    const int px0 = w_pos & 0xFF, py0 = (w_pos >> 8) & 0xFF;
    int px = px0, py = py0, dir = (w_pos >> 16) & 0xFF, sleeping = (w_pos >> 24) & 0xFF;
    const uint32_t win_key = 0x80000000u | (w_pos & 0xFFFFu);
    int a = ((unsigned)action < (unsigned)AC_COUNT) ? action : (int)AC_NOOP;
    if (sleeping) a = AC_NOOP;
    // a kept window serves later steps with other actions: it is always loaded whole
    const WinRect loaded = KEEP_WIN ? full_window() : window_for_action(a);
    if (!KEEP_WIN || e[LDS_WINPOS] != win_key) load_window<G>(l, px0, py0, map, e + LDS_WIN, loaded);
    // where a lane with nothing to read points its load: the player's own cell, whose cache line
    // the window load fetches anyway (any other fixed cell would cost a line of its own)
    const int idle_cell = map_index(px0, py0);
    const int woff = (px0 - WIN_COLS / 2) & 3;      // where window column 0 sits in a row
    int vit[4], cnt[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { vit[i] = (w_vit >> (4 * i)) & 15; cnt[i] = (int)(int8_t)(w_cnt >> (8 * i)); }
    uint32_t phase = w_vit >> 16;
    uint32_t ach = rec[RW_ACH];
    const uint32_t t = rec[RW_T], episode = rec[RW_EPISODE], seed_lo = rec[RW_SEED_LO], seed_hi = rec[RW_SEED_HI];
    static_assert(G % 4 == 0, "a lane's slots must share one Philox block");
    const U4 dr = philox4x32_10(env, t, episode, (DOM_STEP << 16) | (uint32_t)(l & 3), seed_lo, seed_hi);
    uint32_t mw[NSM];                // mob words of the slots this lane owns
    uint32_t sw[NSM];                // their packed draws
#pragma unroll
    for (int s = 0; s < NSM; ++s) {
        const int k = l + s * G;
        mw[s] = k < NMOB ? rec[RW_MOB + k] : 0u;
        const int w = k >> 2;
        sw[s] = w == 0 ? dr.w[0] : (w == 1 ? dr.w[1] : (w == 2 ? dr.w[2] : 0u));
    }
    uint32_t qw[NSP];                // plant words
    int q_block[NSP];
#pragma unroll
    for (int s = 0; s < NSP; ++s) {
        const int k = l + s * G;
        qw[s] = k < NPLANT ? rec[RW_PLANT + k] : 0u;
        q_block[s] = (int)map[(qw[s] & 1u) ? map_index(mob_x(qw[s]), mob_y(qw[s])) : idle_cell];   // unconditional load
        if (!(qw[s] & 1u)) q_block[s] = BK_INVALID;
    }
    const int health0 = vit[0];
    const uint32_t ach0 = ach;
    const uint32_t sapling_draw = (uint32_t)Gr::shfl((int)dr.w[3], 3);

    group_sync();   // the window is in LDS
    if (KEEP_WIN && l == 0) e[LDS_WINPOS] = win_key;

    // ---- phase 1: the player's action ----------------------------------------------------------
    bool l_table = false, l_furnace = false;
#pragma unroll
    for (int it = 0; it < (9 + G - 1) / G; ++it) {
        const int j = l + it * G;
        if (j >= 9) break;
        const int b = win[CX_IDX((3 + j / 3) * WIN_PITCH + woff + 4 + j % 3, WIN_ROWS * WIN_PITCH)];
        l_table = l_table || b == BK_TABLE;
        l_furnace = l_furnace || b == BK_FURNACE;
    }
    const bool is_move = a >= AC_LEFT && a <= AC_DOWN;
    if (is_move) dir = a;
    const int ddx = dir_dx(dir), ddy = dir_dy(dir);
    const int fx = px + ddx, fy = py + ddy;
    const bool f_in = in_map(fx, fy);
    const uint32_t fkey = cell_key(fx, fy);
    const int f_win = (WIN_ROWS / 2 + ddy) * WIN_PITCH + woff + WIN_COLS / 2 + ddx;
    const int fb = win[CX_IDX(f_win, WIN_ROWS * WIN_PITCH)];
    // which mob (if any) stands on the facing cell: owner lane, sub-slot and hp
    int my_hit = -1;
    uint32_t plant_alive = 0;
#pragma unroll
    for (int s = 0; s < NSM; ++s)
        if ((mw[s] & KEY_MASK) == fkey) my_hit = s | (int)(__builtin_amdgcn_ubfe(mw[s], 16, 4) << 4);
    const uint32_t hit_lanes = Gr::ballot(my_hit >= 0);
    const int hit_lane = hit_lanes ? (__ffs((int)hit_lanes) - 1) : 0;
    const int hit_info = Gr::shfl(my_hit, hit_lane);
    const int hit = hit_lanes ? hit_lane + G * (hit_info & 15) : -1;   // mob slot index
    const int hit_hp = hit_info >> 4;

    int modval = -1;                 // new block of the facing cell, if the action edits it
    bool ate_ripe = false;
    int new_plant_slot = -1;

    if (is_move) {
        if (f_in && hit < 0) {
            if (walkable_ground(fb)) { px = fx; py = fy; }
            else if (fb == BK_LAVA) { px = fx; py = fy; vit[0] = 0; }
        }
    } else if (a == AC_DO) {
        if (f_in) {
            if (hit >= 0) {
                const int type = (hit * 11) >> 5;
                if (type != MT_ARROW) {
                    const int dmg = (w_inv & (1u << 29)) ? 5 : ((w_inv & (1u << 28)) ? 3 : ((w_inv & (1u << 27)) ? 2 : 1));
                    const int hp = hit_hp - dmg;
#pragma unroll
                    for (int s = 0; s < NSM; ++s)
                        if (l + s * G == hit) mw[s] = hp > 0 ? ((mw[s] & ~(15u << 16)) | ((uint32_t)hp << 16)) : 0u;
                    if (hp <= 0) {
                        if (type == MT_ZOMBIE) ach |= 1u << ACH_DEFEAT_ZOMBIE;
                        if (type == MT_SKELETON) ach |= 1u << ACH_DEFEAT_SKELETON;
                        if (type == MT_COW) {
                            vit[1] = min(MAX_COUNT, vit[1] + FOOD_COW);
                            cnt[0] = 0;
                            ach |= 1u << ACH_EAT_COW;
                        }
                    }
                }
            } else if (fb == BK_WATER) {
                vit[2] = min(MAX_COUNT, vit[2] + 1); cnt[1] = 0; ach |= 1u << ACH_COLLECT_DRINK;
            } else if (fb == BK_RIPE) {
                vit[1] = min(MAX_COUNT, vit[1] + FOOD_PLANT); cnt[0] = 0; ach |= 1u << ACH_EAT_PLANT;
                modval = BK_PLANT;
                ate_ripe = true;
            } else if (fb <= BK_DIAMOND) {
                const int item1 = (int)((DO_ITEM >> (4 * fb)) & 15u);        // item + 1
                const int tool = (int)((DO_GATE >> (2 * fb)) & 3u);
                const bool gate = tool ? ((w_inv >> (23 + tool)) & 1u) : (fb != BK_GRASS || sapling_draw < P_SAPLING);
                const int sh = item1 ? 4 * (item1 - 1) : 0;
                if (item1 && gate && ((w_inv >> sh) & 15u) < (uint32_t)MAX_COUNT) {
                    w_inv += 1u << sh;
                    ach |= 1u << (uint32_t)((DO_ACH >> (5 * fb)) & 31u);
                    if ((MINED_MASK >> fb) & 1u) modval = BK_PATH;
                }
            }
        }
    } else if (a == AC_SLEEP) {
        if (vit[3] < MAX_COUNT) sleeping = 1;
    } else if (a >= AC_PLACE_STONE && a <= AC_PLACE_PLANT) {
        if (f_in && hit < 0) {
            const bool ground = walkable_ground(fb);
            if (a == AC_PLACE_STONE) {
                if ((w_inv & 0xF0u) && (ground || fb == BK_WATER || fb == BK_LAVA)) {
                    w_inv -= 0x10u; modval = BK_STONE; ach |= 1u << ACH_PLACE_STONE;
                }
            } else if (a == AC_PLACE_TABLE) {
                if ((w_inv & 0xFu) && ground) { w_inv -= 0x1u; modval = BK_TABLE; ach |= 1u << ACH_PLACE_TABLE; }
            } else if (a == AC_PLACE_FURNACE) {
                if ((w_inv & 0xF0u) && ground && Gr::ballot(l_table) != 0) {
                    w_inv -= 0x10u; modval = BK_FURNACE; ach |= 1u << ACH_PLACE_FURNACE;
                }
            } else {
#pragma unroll
                for (int s = 0; s < NSP; ++s) plant_alive |= Gr::ballot(qw[s] & 1u) << (s * G);
                const uint32_t free_slots = ~plant_alive & ((1u << p.cap_plant) - 1u);
                if ((w_inv & 0xF00000u) && fb == BK_GRASS && free_slots) {
                    w_inv -= 0x100000u; modval = BK_PLANT; ach |= 1u << ACH_PLACE_PLANT;
                    new_plant_slot = __ffs((int)free_slots) - 1;
                }
            }
        }
    } else if (a >= AC_MAKE_WOOD_PICKAXE) {
        const int which = a - AC_MAKE_WOOD_PICKAXE;               // 0..5: pickaxes then swords
        const int tier = which >= 3 ? which - 3 : which;          // 0 wood, 1 stone, 2 iron
        // cost in the inventory's nibble layout: wood | stone<<4 | coal<<8 | iron<<12
        const uint32_t cost = tier == 0 ? 0x0001u : (tier == 1 ? 0x0011u : 0x1101u);
        const uint32_t nonzero = (w_inv | (w_inv >> 1) | (w_inv >> 2) | (w_inv >> 3)) & 0x1111u;
        const bool near_table = Gr::ballot(l_table) != 0, near_furnace = Gr::ballot(l_furnace) != 0;
        const bool ok = !((w_inv >> (24 + which)) & 1u) && near_table && (tier != 2 || near_furnace) && (nonzero & cost) == cost;
        if (ok) {
            w_inv = (w_inv - cost) | (1u << (24 + which));
            ach |= 1u << ((MAKE_ACH >> (5 * which)) & 31u);
        }
    }
    const int modcell = modval >= 0 ? fy * MAPW + fx : -1;
    if (modval >= 0) {
        if (l == 0) { map[map_index(fx, fy)] = (uint8_t)modval; win[CX_IDX(f_win, WIN_ROWS * WIN_PITCH)] = (uint8_t)modval; }
#pragma unroll
        for (int s = 0; s < NSP; ++s) {
            const int k = l + s * G;
            if (k == new_plant_slot) { qw[s] = fkey; q_block[s] = BK_PLANT; }
            else if ((qw[s] & KEY_MASK) == fkey) { q_block[s] = modval; if (ate_ripe) qw[s] &= 0xFFFFu; }
        }
    }
    const int mvx = px - px0, mvy = py - py0;
    const uint32_t pkey = cell_key(px, py);

    // ---- phase 2: mobs.  Intent of each slot from its own state, the player and its draws ----
    // packed intent: kind | ok<<3 | at_player<<4 | target key<<8 | direction<<24
    int packed[NSM];
    int n_attack = 0, n_arrow = 0;
    int kind_[NSM], ndir_[NSM], tx_[NSM], ty_[NSM], tb_[NSM];
#pragma unroll
    for (int s = 0; s < NSM; ++s) {
        const int k = l + s * G;
        int kind = K_NONE, ndir = 0;
        const int mx = mob_x(mw[s]), my = mob_y(mw[s]);
        if (mw[s] & 1u) {
            const int type = (k * 11) >> 5;
            const int dx = px - mx, dy = py - my;
            const int adx = iabs(dx), ady = iabs(dy), cheb = max(adx, ady);
            const uint32_t m8 = (sw[s] >> 16) & 7u;               // movement choice
            const uint32_t r_act = sw[s] & 0xFFFFu;               // decision draw
            const int toward = adx >= ady ? (dx < 0 ? 1 : 2) : (dy < 0 ? 3 : 4);
            const int wander = m8 < 4 ? (int)m8 + 1 : 0;
            const int cd = (int)__builtin_amdgcn_ubfe(mw[s], 20, 4);
            if (type == MT_ZOMBIE || type == MT_SKELETON) { if (cd > 0) mw[s] -= 1u << 20; }
            const bool ready = cd <= 1;                            // cooldown is zero after the decrement
            if (type == MT_ZOMBIE) {
                if (adx + ady == 1) {
                    if (ready) { kind = K_ATTACK; mw[s] = (mw[s] & ~(15u << 20)) | ((uint32_t)CD_ZOMBIE << 20); }
                } else {
                    ndir = (cheb < CHASE_RANGE && r_act < P_CHASE) ? toward : wander;
                    if (ndir) kind = K_MOVE;
                }
            } else if (type == MT_COW) {
                ndir = wander;
                if (ndir) kind = K_MOVE;
            } else if (type == MT_SKELETON) {
                const bool aligned = (dx == 0 || dy == 0) && cheb <= SHOOT_RANGE;
                if (aligned && ready && r_act < P_SHOOT) {
                    kind = K_SHOOT; ndir = toward; mw[s] = (mw[s] & ~(15u << 20)) | ((uint32_t)CD_SKELETON << 20);
                } else {
                    ndir = wander ? wander : (cheb <= SHOOT_RANGE ? toward : 0);
                    if (ndir) kind = K_MOVE_PATH;
                }
            } else {
                kind = K_FLY; ndir = (int)__builtin_amdgcn_ubfe(mw[s], 13, 3);
            }
        }
        kind_[s] = kind; ndir_[s] = ndir;
        tx_[s] = mx + dir_dx(ndir); ty_[s] = my + dir_dy(ndir);
        // terrain of the target cell: loaded unconditionally (the idle cell when there is no target)
        const bool need = kind != K_NONE && kind != K_ATTACK && in_map(tx_[s], ty_[s]);
        tb_[s] = (int)map[need ? map_index(tx_[s], ty_[s]) : idle_cell];
    }
    // spawn candidates (phase 3) are fixed by the draws and the player's position: read their
    // terrain now so the loads overlap the mob resolution below
    uint32_t sp_key[3];
    int sp_b[3];
    bool sp_cand[3];
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        const uint32_t sp_w = (uint32_t)Gr::shfl((int)dr.w[3], j);              // misc[j]
        const int dx = (int)(((sp_w & 1023u) * 31u) >> 10) - 15;
        const int dy = (int)((((sp_w >> 10) & 1023u) * 31u) >> 10) - 15;
        const uint32_t sp_p = sp_w >> 20;
        const uint32_t thr = j == 0 ? luts->zombie_thr[phase] >> 20 : (j == 1 ? P_COW_SPAWN : P_SKELETON_SPAWN);
        const int sx = px + dx, sy = py + dy;
        // a candidate only if the probability draw passes too: most attempts end here, and the
        // terrain byte (a whole cache line of traffic) is then not fetched at all
        sp_cand[j] = max(iabs(dx), iabs(dy)) >= SPAWN_MIN_DIST && in_map(sx, sy) && sp_p < thr;
        sp_key[j] = cell_key(sx & 63, sy & 63);
        sp_b[j] = (int)map[sp_cand[j] ? map_index(sx, sy) : idle_cell];
        if (!sp_cand[j]) sp_b[j] = BK_OOB;
    }
#pragma unroll
    for (int s = 0; s < NSM; ++s) {
        const int kind = kind_[s], tx = tx_[s], ty = ty_[s];
        const bool t_in = in_map(tx, ty);
        int tb = (kind != K_NONE && kind != K_ATTACK && t_in) ? tb_[s] : (int)BK_OOB;
        if (ty * MAPW + tx == modcell && t_in) tb = modval;
        const uint32_t tkey = cell_key(tx & 63, ty & 63);
        const bool at_player = t_in && tkey == pkey;
        const bool t_ok = t_in && (kind == K_MOVE ? walkable_ground(tb) : (kind == K_MOVE_PATH ? tb == BK_PATH : arrow_flyable(tb)));
        packed[s] = kind | ((int)t_ok << 3) | ((int)at_player << 4) | (int)(tkey << 8) | (ndir_[s] << 24);
        n_attack += __popc(Gr::ballot(kind == K_ATTACK));
        n_arrow += __popc(Gr::ballot((kind == K_SHOOT || kind == K_FLY) && at_player));
    }

    const int damage = n_attack * (sleeping ? DMG_ZOMBIE_SLEEP : DMG_ZOMBIE) + n_arrow * DMG_ARROW;

    // Moves resolve one slot at a time in the order zombies, cows, arrows, skeletons; each sees
    // the positions left by the slots before it.  An arrow shot now first flies next step.
    // The slot index is a compile-time constant here, so each iteration only carries the code
    // of its own mob type, and a wave-wide vote skips slots that are idle in all its groups.
    constexpr int ORDER[NMOB] = { 0, 1, 2, 3, 4, 5, 9, 10, 11, 6, 7, 8 };
#pragma unroll
    for (int i = 0; i < NMOB; ++i) {
        const int k = ORDER[i];
        const int ks = k / G, kl = k % G;           // owner sub-slot and lane (compile-time)
        const int ik = Gr::shfl(packed[ks], kl);
        const int kk = ik & 7;
        if (!__any(kk != K_NONE && kk != K_ATTACK)) continue;
        const bool k_ok = (ik >> 3) & 1, k_at = (ik >> 4) & 1;
        const uint32_t tkey = ((uint32_t)ik >> 8) & KEY_MASK;
        bool l_occ = false;
#pragma unroll
        for (int s = 0; s < NSM; ++s) l_occ = l_occ || (mw[s] & KEY_MASK) == tkey;
        const bool blocked = Gr::ballot(l_occ) != 0 || k_at || !k_ok;
        if (k < 6 || (k < 9 && kk == K_MOVE_PATH)) {
            if ((kk == K_MOVE || kk == K_MOVE_PATH) && !blocked && l == kl) mw[ks] = mob_moved(mw[ks], tkey);
        } else if (k < 9) {
            if (kk == K_SHOOT && !blocked) {
                const uint32_t arrows = (Gr::ballot(mw[9 / G] & 1u) >> (9 % G)) & 7u;   // bit j = arrow slot 9+j alive
                const uint32_t free_arrows = ~arrows & ((1u << p.cap_arrow) - 1u) & 7u;
                if (free_arrows) {
                    const int ka = 9 + __ffs((int)free_arrows) - 1;
                    if (l == ka % G) mw[9 / G] = tkey | ((uint32_t)((ik >> 24) & 7) << 13);
                }
            }
        } else {
            if (kk == K_FLY && l == kl) mw[ks] = blocked ? 0u : mob_moved(mw[ks], tkey);
        }
    }
    vit[0] = max(0, vit[0] - damage);

    // ---- phase 3: despawn far mobs, then one spawn attempt per type -----------------------------
#pragma unroll
    for (int s = 0; s < NSM; ++s)
        if ((mw[s] & 1u) && max(iabs(mob_x(mw[s]) - px), iabs(mob_y(mw[s]) - py)) > DESPAWN_DIST) mw[s] = 0u;
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        uint32_t taken = 0;                          // bit i = slot 3j+i alive
        bool l_occ = false;
#pragma unroll
        for (int s = 0; s < NSM; ++s) l_occ = l_occ || (mw[s] & KEY_MASK) == sp_key[j];
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const int ss = (3 * j + i) / G, sl = (3 * j + i) % G;
            taken |= ((Gr::ballot(mw[ss] & 1u) >> sl) & 1u) << i;
        }
        const bool occ = Gr::ballot(l_occ) != 0;
        const uint32_t cap = j == 0 ? p.cap_zombie : (j == 1 ? p.cap_cow : p.cap_skeleton);
        const uint32_t free_slots = ~taken & ((1u << cap) - 1u) & 7u;
        const int want = j == 2 ? BK_PATH : BK_GRASS;
        if (sp_cand[j] && free_slots && !occ && sp_b[j] == want) {
            const int kn = 3 * j + __ffs((int)free_slots) - 1;
            const uint32_t hp = j == 0 ? HP_ZOMBIE : (j == 1 ? HP_COW : HP_SKELETON);
#pragma unroll
            for (int s = 0; s < NSM; ++s)
                if (l + s * G == kn) mw[s] = sp_key[j] | (hp << 16);
        }
    }

    // ---- phase 4: plants ----------------------------------------------------------------------------
    bool any_plant = false;
#pragma unroll
    for (int s = 0; s < NSP; ++s) any_plant = any_plant || (qw[s] & 1u);
    if (__any(any_plant)) {                          // skipped by waves that track no plant at all
        uint32_t zw[3];
#pragma unroll
        for (int z = 0; z < 3; ++z) zw[z] = (uint32_t)Gr::shfl((int)mw[z / G], z % G);
#pragma unroll
        for (int s = 0; s < NSP; ++s) {
            if (!(qw[s] & 1u)) continue;
            const int qx = mob_x(qw[s]), qy = mob_y(qw[s]);
            bool zombie_near = false;
#pragma unroll
            for (int z = 0; z < 3; ++z)
                zombie_near = zombie_near || ((zw[z] & 1u) && iabs(mob_x(zw[z]) - qx) + iabs(mob_y(zw[z]) - qy) == 1);
            if ((qw[s] >> 16) < 65535u) qw[s] += 1u << 16;
            int nb = q_block[s];
            if (nb == BK_PLANT && (qw[s] >> 16) >= (uint32_t)RIPE_AGE) nb = BK_RIPE;
            if (zombie_near && ((sw[s] >> 19) & 0xFFu) < P_PLANT_EATEN) nb = BK_GRASS;
            if (nb != q_block[s]) {
                map[map_index(qx, qy)] = (uint8_t)nb;
                const int wx = qx - (px0 - WIN_COLS / 2), wy = qy - (py0 - WIN_ROWS / 2);
                if ((unsigned)wx < (unsigned)WIN_COLS && (unsigned)wy < (unsigned)WIN_ROWS) win[CX_IDX(wy * WIN_PITCH + woff + wx, WIN_ROWS * WIN_PITCH)] = (uint8_t)nb;
            }
            if (nb == BK_GRASS) qw[s] = 0u;
        }
    }

    // ---- phase 5: needs ------------------------------------------------------------------------------
    {
        const int asleep = sleeping;
        cnt[0] += asleep ? 1 : 2;
        if (cnt[0] > 50) { cnt[0] = 0; vit[1] = max(0, vit[1] - 1); }
        cnt[1] += asleep ? 1 : 2;
        if (cnt[1] > 40) { cnt[1] = 0; vit[2] = max(0, vit[2] - 1); }
        if (asleep) {
            cnt[2]--;
            if (cnt[2] < -10) { cnt[2] = 0; vit[3] = min(MAX_COUNT, vit[3] + 1); }
        } else {
            cnt[2]++;
            if (cnt[2] > 30) { cnt[2] = 0; vit[3] = max(0, vit[3] - 1); }
        }
        if (vit[0] > 0) {
            const bool fed = vit[1] > 0 && vit[2] > 0 && (vit[3] > 0 || asleep);
            cnt[3] += fed ? (asleep ? 4 : 2) : (asleep ? -1 : -2);
            if (cnt[3] > 50) { cnt[3] = 0; vit[0] = min(MAX_COUNT, vit[0] + 1); }
            if (cnt[3] < -30) { cnt[3] = 0; vit[0]--; }
        }
        if (asleep && (vit[3] >= MAX_COUNT || damage > 0)) { sleeping = 0; ach |= 1u << ACH_WAKE_UP; }
    }

    // ---- reward, time, done ---------------------------------------------------------------------------
    StepOut out;
    out.mvx = mvx; out.mvy = mvy; out.woff = woff;
    out.unlocked = ach & ~ach0;
    const int gained = __popc(out.unlocked);
    out.reward = (float)(10 * gained + (vit[0] - health0)) * 0.1f;
    const uint32_t t1 = t + 1;
    phase = phase + 1 == p.day_length ? 0u : phase + 1;
    out.done = vit[0] <= 0 || t1 >= p.max_episode_steps;
    if (out.done) return out;

    // ---- pack the record back into LDS ------------------------------------------------------------------
    group_sync();
    if (l == 0) {
        rec[RW_POS] = (uint32_t)px | ((uint32_t)py << 8) | ((uint32_t)dir << 16) | ((uint32_t)sleeping << 24);
        rec[RW_INV] = w_inv;
        rec[RW_VIT] = (uint32_t)vit[0] | ((uint32_t)vit[1] << 4) | ((uint32_t)vit[2] << 8) | ((uint32_t)vit[3] << 12) | (phase << 16);
        rec[RW_CNT] = (uint32_t)(cnt[0] & 0xFF) | ((uint32_t)(cnt[1] & 0xFF) << 8) | ((uint32_t)(cnt[2] & 0xFF) << 16) | ((uint32_t)(cnt[3] & 0xFF) << 24);
        rec[RW_ACH] = ach;
        rec[RW_T] = t1;
    }
#pragma unroll
    for (int s = 0; s < NSM; ++s) {
        const int k = l + s * G;
        if (k < NMOB) rec[RW_MOB + k] = mw[s];
    }
#pragma unroll
    for (int s = 0; s < NSP; ++s) {
        const int k = l + s * G;
        if (k < NPLANT) rec[RW_PLANT + k] = qw[s];
    }
    group_sync();
    return out;
}

}  // namespace cx
