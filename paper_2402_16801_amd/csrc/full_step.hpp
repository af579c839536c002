// One step of one full-Craftax environment by one wavefront.
//
// The player's state is unpacked into wave-uniform scalars (every lane computes the same
// values, so the compiler keeps them in scalar registers and branches on them without
// divergence); lane k < 14 holds mob slot k of the current floor, lane k < 10 plant slot k.
// The phases follow section "Craftax: An Extension of Crafter ..." for what exists (floors,
// ladders, combat with three damage elements, bow, spells, potions, enchanting, attributes,
// boss waves); their order and every constant are this library's own frozen reading:
// action -> mobs (melee, passive, mob projectiles, player projectiles, ranged) -> despawn /
// spawn -> plants -> needs -> reward, done.
#pragma once

#include "full_common.hpp"

namespace cf {

struct Player {
    int px, py, dir, floor;
    int sleeping, resting, fireball, iceball, book, pickaxe, sword, sword_ench, bow, bow_ench, boss_vulnerable, boss_hits;
    uint32_t armour, armour_ench;      // 4 x 2 bits each
    int xp, dex, str, intel;
    int inv[10];
    uint64_t potion;                   // 6 bytes
    int vit[5], cnt[5];
    int phase;
    uint32_t perm;
    int visited;
    uint64_t kills07;                  // floors 0..7, a byte each
    int kills8;
    uint32_t ach[3];
    uint32_t t, episode;
};

__device__ inline int sext8(uint32_t v) { return (int)(int8_t)(v & 0xFFu); }

template <int GW = 64>
__device__ __forceinline__ void unpack_player(const uint32_t* rec, Player& P)
{
    using G = Lanes<GW>;
    const uint32_t r0 = G::uniu(rec[R_POS]), r1 = G::uniu(rec[R_FLAGS]), r2 = G::uniu(rec[R_ATTR]);
    P.px = r0 & 0xFF; P.py = (r0 >> 8) & 0xFF; P.dir = (r0 >> 16) & 0xFF; P.floor = (r0 >> 24) & 0xF;
    P.sleeping = r1 & 1; P.resting = (r1 >> 1) & 1; P.fireball = (r1 >> 2) & 1; P.iceball = (r1 >> 3) & 1;
    P.book = (r1 >> 4) & 3; P.pickaxe = (r1 >> 6) & 7; P.sword = (r1 >> 9) & 7; P.sword_ench = (r1 >> 12) & 3;
    P.bow = (r1 >> 14) & 1; P.bow_ench = (r1 >> 15) & 3; P.boss_vulnerable = (r1 >> 17) & 1; P.boss_hits = (r1 >> 18) & 15;
    P.armour = r2 & 0xFF; P.armour_ench = (r2 >> 8) & 0xFF;
    P.xp = (r2 >> 16) & 15; P.dex = (r2 >> 20) & 7; P.str = (r2 >> 23) & 7; P.intel = (r2 >> 26) & 7;
    const uint32_t i0 = G::uniu(rec[R_INV]), i1 = G::uniu(rec[R_INV + 1]), i2 = G::uniu(rec[R_INV + 2]), i3 = G::uniu(rec[R_POT]);
#pragma unroll
    for (int i = 0; i < 4; ++i) { P.inv[i] = (i0 >> (8 * i)) & 0xFF; P.inv[4 + i] = (i1 >> (8 * i)) & 0xFF; }
    P.inv[8] = i2 & 0xFF; P.inv[9] = (i2 >> 8) & 0xFF;
    P.potion = (uint64_t)(i2 >> 16) | ((uint64_t)i3 << 16);
    const uint32_t v0 = G::uniu(rec[R_VIT]), v1 = G::uniu(rec[R_MANA]), c0 = G::uniu(rec[R_CNT]);
#pragma unroll
    for (int i = 0; i < 4; ++i) { P.vit[i] = (v0 >> (8 * i)) & 0xFF; P.cnt[i] = sext8(c0 >> (8 * i)); }
    P.vit[V_MANA] = v1 & 0xFF; P.cnt[K_MANA] = sext8(v1 >> 8); P.phase = (int)(v1 >> 16);
    const uint32_t pm = G::uniu(rec[R_PERM]);
    P.perm = pm & 0x3FFFFu; P.visited = (pm >> 18) & 0x1FF;
    P.kills07 = (uint64_t)G::uniu(rec[R_KILLS]) | ((uint64_t)G::uniu(rec[R_KILLS + 1]) << 32);
    P.kills8 = G::uniu(rec[R_KILLS + 2]) & 0xFF;
#pragma unroll
    for (int i = 0; i < 3; ++i) P.ach[i] = G::uniu(rec[R_ACH + i]);
    P.t = G::uniu(rec[R_T]); P.episode = G::uniu(rec[R_EPISODE]);
}

// packs everything that can change back into the LDS copy of the record (one lane writes)
__device__ __forceinline__ void pack_player(uint32_t* rec, const Player& P)
{
    rec[R_POS] = (uint32_t)P.px | ((uint32_t)P.py << 8) | ((uint32_t)P.dir << 16) | ((uint32_t)P.floor << 24);
    rec[R_FLAGS] = (uint32_t)P.sleeping | ((uint32_t)P.resting << 1) | ((uint32_t)P.fireball << 2) | ((uint32_t)P.iceball << 3) |
                   ((uint32_t)P.book << 4) | ((uint32_t)P.pickaxe << 6) | ((uint32_t)P.sword << 9) | ((uint32_t)P.sword_ench << 12) |
                   ((uint32_t)P.bow << 14) | ((uint32_t)P.bow_ench << 15) | ((uint32_t)P.boss_vulnerable << 17) | ((uint32_t)P.boss_hits << 18);
    rec[R_ATTR] = P.armour | (P.armour_ench << 8) | ((uint32_t)P.xp << 16) | ((uint32_t)P.dex << 20) | ((uint32_t)P.str << 23) | ((uint32_t)P.intel << 26);
    rec[R_INV] = (uint32_t)P.inv[0] | ((uint32_t)P.inv[1] << 8) | ((uint32_t)P.inv[2] << 16) | ((uint32_t)P.inv[3] << 24);
    rec[R_INV + 1] = (uint32_t)P.inv[4] | ((uint32_t)P.inv[5] << 8) | ((uint32_t)P.inv[6] << 16) | ((uint32_t)P.inv[7] << 24);
    rec[R_INV + 2] = (uint32_t)P.inv[8] | ((uint32_t)P.inv[9] << 8) | ((uint32_t)(P.potion & 0xFFFFu) << 16);
    rec[R_POT] = (uint32_t)(P.potion >> 16);
    rec[R_VIT] = (uint32_t)P.vit[0] | ((uint32_t)P.vit[1] << 8) | ((uint32_t)P.vit[2] << 16) | ((uint32_t)P.vit[3] << 24);
    rec[R_MANA] = (uint32_t)P.vit[V_MANA] | ((uint32_t)(P.cnt[K_MANA] & 0xFF) << 8) | ((uint32_t)P.phase << 16);
    rec[R_CNT] = (uint32_t)(P.cnt[0] & 0xFF) | ((uint32_t)(P.cnt[1] & 0xFF) << 8) | ((uint32_t)(P.cnt[2] & 0xFF) << 16) | ((uint32_t)(P.cnt[3] & 0xFF) << 24);
    rec[R_PERM] = P.perm | ((uint32_t)P.visited << 18);
    rec[R_KILLS] = (uint32_t)P.kills07; rec[R_KILLS + 1] = (uint32_t)(P.kills07 >> 32); rec[R_KILLS + 2] = (uint32_t)P.kills8;
    rec[R_ACH] = P.ach[0]; rec[R_ACH + 1] = P.ach[1]; rec[R_ACH + 2] = P.ach[2];
    rec[R_T] = P.t; rec[R_EPISODE] = P.episode;
}

__device__ inline int get_kills(const Player& P, int f) { return f < 8 ? (int)((P.kills07 >> (8 * f)) & 0xFF) : P.kills8; }
__device__ inline int get_potion(const Player& P, int c) { return (int)((P.potion >> (8 * c)) & 0xFF); }
__device__ inline void set_potion(Player& P, int c, int v) { P.potion = (P.potion & ~(0xFFull << (8 * c))) | ((uint64_t)v << (8 * c)); }
__device__ inline void unlock(Player& P, int a)
{
    const uint32_t bit = 1u << (a & 31);
    const int w = a >> 5;
    P.ach[0] |= w == 0 ? bit : 0u; P.ach[1] |= w == 1 ? bit : 0u; P.ach[2] |= w == 2 ? bit : 0u;
}
__device__ inline int cap_health(const Player& P) { return 9 + (5 * (P.str - 1)) / 4; }
__device__ inline int cap_need(const Player& P) { return 9 + 2 * (P.dex - 1); }
__device__ inline int cap_mana(const Player& P) { return 9 + 3 * (P.intel - 1); }
__device__ inline int toward(int dx, int dy) { return iabs(dx) >= iabs(dy) ? (dx < 0 ? 1 : 2) : (dy < 0 ? 3 : 4); }
// damage after defence: every element is reduced by its own percentage, integer parts
__device__ inline int through(int ap, int af, int ai, int dp, int df, int di)
{
    return ap * (100 - dp) / 100 + af * (100 - df) / 100 + ai * (100 - di) / 100;
}

// Loads the 11 x 13 window of floor f centred on (cx, cy) into LDS (both maps).
template <int GW = 64>
__device__ __forceinline__ void load_window(int l, const uint8_t* __restrict__ maps, int f, int cx_, int cy_, uint8_t* wb, uint8_t* wi)
{
#pragma unroll
    for (int it = 0; it < (WIN_ROWS * WIN_COLS + GW - 1) / GW; ++it) {
        const int i = l + GW * it;
        if (i < WIN_ROWS * WIN_COLS) {
            const int r = i / WIN_COLS, c = i - r * WIN_COLS;
            const int x = cx_ - WIN_COLS / 2 + c, y = cy_ - WIN_ROWS / 2 + r;
            int b = B_OOB, il = MAX_LIGHT << 3;
            if (inb(x, y)) { b = maps[block_off(f, x, y)]; il = maps[il_off(f, x, y)]; }
            wb[CX_IDX(r * WIN_PITCH + c, WIN_ROWS * WIN_PITCH)] = (uint8_t)b;
            wi[CX_IDX(r * WIN_PITCH + c, WIN_ROWS * WIN_PITCH)] = (uint8_t)il;
        }
    }
}

struct MobRegs { int alive, x, y, dir, hp, cd, type; };
__device__ inline void clear_mob(MobRegs& m) { m.alive = m.x = m.y = m.dir = m.hp = m.cd = m.type = 0; }

struct StepOut { bool done; float reward; int wx0, wy0; uint32_t unlocked[3]; };   // unlocked: achievement bits new after this step

enum Intent : int { N_NONE = 0, N_DAMAGE, N_DAMAGE_DIE, N_DIE, N_MOVE, N_SHOOT, N_FLY, N_PPROJ };

// e: this wave's LDS area with the record loaded.  genv: the environment's 1024-byte block in
// HBM.  maps: its floors.  m, qw: this lane's mob slot (current floor) and plant word.
// after_load: called once the loads of the current window have been issued and stored, before the
// wave waits for them (the caller parks data it fetched earlier there).
template <int GW = 64, typename AfterLoad>
__device__ __forceinline__ StepOut step_env(const int l, const uint32_t env, uint32_t* e, uint32_t* __restrict__ genv,
                                   uint8_t* __restrict__ maps, const Luts* __restrict__ luts, const int action_in,
                                   const Params& p, MobRegs& m, uint32_t& qw, Player& P, AfterLoad&& after_load)
{
    using G = Lanes<GW>;
    uint32_t* rec = e + L_REC;
    uint8_t* wb = reinterpret_cast<uint8_t*>(e + L_WB);
    uint8_t* wi = reinterpret_cast<uint8_t*>(e + L_WI);
    unpack_player<GW>(rec, P);
    // asked for now, needed in the spawn phase: by then it has long arrived
    const uint32_t zombie_thr = luts->zombie_thr[P.phase];
    const uint32_t seed_lo = G::uniu(rec[R_SEED_LO]), seed_hi = G::uniu(rec[R_SEED_HI]);

    // this step's draws: lane k computes Philox block k = (move k, decision k, plant-eaten k, misc k)
    const U4 rnd = philox4x32_10(env, P.t, P.episode, (cx::DOM_STEP << 16) | (uint32_t)(l < NSLOT ? l : 0), seed_lo, seed_hi);
    uint32_t misc[12];
#pragma unroll
    for (int i = 0; i < 12; ++i) misc[i] = (uint32_t)G::get((int)rnd.w[3], i);

    // mob table of the current floor and the window around the player
    {
        const uint32_t w = l < NSLOT ? genv[REC_DWORDS + P.floor * MOBTAB_DWORDS + l] : 0u;
        const Mob u = unpack_mob(w);
        m.alive = u.alive; m.x = u.x; m.y = u.y; m.dir = u.dir; m.hp = u.hp; m.cd = u.cd; m.type = u.type;
    }
    qw = l < NPLANT ? rec[R_PLANT + l] : 0u;
    int q_alive = qw & 1u, q_x = (qw >> 1) & 63u, q_y = (qw >> 7) & 63u, q_age = (int)(qw >> 16);
    // block under every plant (floor 0), fetched before anything is stored this step
    int q_block = B_INVALID;
    if (q_alive) q_block = maps[block_off(0, q_x, q_y)];
    int wx0 = P.px - WIN_COLS / 2, wy0 = P.py - WIN_ROWS / 2;
    load_window<GW>(l, maps, P.floor, P.px, P.py, wb, wi);
    after_load();
    wave_sync();

    auto win_b = [&](int x, int y) { return G::uni((int)wb[CX_IDX((y - wy0) * WIN_PITCH + (x - wx0), WIN_ROWS * WIN_PITCH)]); };
    auto win_i = [&](int x, int y) { return G::uni((int)wi[CX_IDX((y - wy0) * WIN_PITCH + (x - wx0), WIN_ROWS * WIN_PITCH)]); };
    auto in_win = [&](int x, int y) { return (unsigned)(x - wx0) < (unsigned)WIN_COLS && (unsigned)(y - wy0) < (unsigned)WIN_ROWS; };
    auto occ_mask = [&](int x, int y) -> uint32_t { return (uint32_t)G::ballot(m.alive && m.x == x && m.y == y); };
    // the one block cell the player may change this step; mobs read their terrain from HBM and
    // take this cell from here instead
    int patch_f = -1, patch_x = -1, patch_y = -1, patch_b = 0;
    auto set_block = [&](int x, int y, int b) {
        if (l == 0) {
            maps[block_off(P.floor, x, y)] = (uint8_t)b;
            if (in_win(x, y)) wb[CX_IDX((y - wy0) * WIN_PITCH + (x - wx0), WIN_ROWS * WIN_PITCH)] = (uint8_t)b;
        }
        wave_sync();
    };
    auto set_facing_block = [&](int x, int y, int b) {
        patch_f = P.floor; patch_x = x; patch_y = y; patch_b = b;
        set_block(x, y, b);
    };
    const int health0 = P.vit[V_HEALTH];
    const uint32_t ach0[3] = { P.ach[0], P.ach[1], P.ach[2] };

    // the player hurts mob slot k; returns true when it died
    auto hurt_mob = [&](int k, int ap, int af, int ai) -> bool {
        if (k >= S_MPROJ0) return false;                       // projectiles cannot be hit
        const int type = G::get(m.type, k), hp = G::get(m.hp, k);
        const CreatureRow c = creature(type);
        const int nhp = hp - through(ap, af, ai, c.Dp, c.Df, c.Di);
        if (nhp > 0) { if (l == k) m.hp = nhp; return false; }
        if (l == k) clear_mob(m);
        unlock(P, c.ach);
        if (k >= S_PASSIVE0) { P.vit[V_FOOD] = min(cap_need(P), P.vit[V_FOOD] + FOOD_MEAT); P.cnt[K_HUNGER] = 0; }
        else {
            const int f = P.floor;
            int kf = get_kills(P, f);
            if (kf < 255) {
                ++kf;
                if (f < 8) P.kills07 = (P.kills07 & ~(0xFFull << (8 * f))) | ((uint64_t)kf << (8 * f));
                else P.kills8 = kf;
            }
            // the way down opens once enough enemies of this floor are gone
            if (f >= 1 && f < FLOORS - 1 && kf >= KILLS_TO_CLEAR) {
                const uint32_t lw = G::uniu(rec[R_LADDER + f]);
                const int lx = (lw >> 16) & 0xFF, ly = (lw >> 24) & 0xFF;
                int il;
                if (in_win(lx, ly)) il = win_i(lx, ly);
                else {
                    __threadfence();                           // a torch placed this step may have lit that cell
                    il = G::uni((int)__hip_atomic_load(maps + il_off(f, lx, ly), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                }
                if ((il & 7) == IT_LADDER_DOWN_BLOCKED) {
                    const int nil = (il & ~7) | IT_LADDER_DOWN;
                    if (l == 0) {
                        maps[il_off(f, lx, ly)] = (uint8_t)nil;
                        if (in_win(lx, ly)) wi[CX_IDX((ly - wy0) * WIN_PITCH + (lx - wx0), WIN_ROWS * WIN_PITCH)] = (uint8_t)nil;
                    }
                    wave_sync();
                }
            }
        }
        return true;
    };
    auto spawn_mob = [&](int slot, int x, int y, int dir, int type, int hp) {
        if (l == slot) { m.alive = 1; m.x = x; m.y = y; m.dir = dir; m.hp = hp; m.cd = 0; m.type = type; }
    };
    auto shot_attack = [&](int kind, int& ap, int& af, int& ai) {
        ap = af = ai = 0;
        if (kind == PP_ARROW) { ap = 2 + (P.dex - 1); if (P.bow_ench == 1) af = 4; if (P.bow_ench == 2) ai = 4; }
        else if (kind == PP_FIREBALL) af = 4 + 2 * (P.intel - 1);
        else ai = 4 + 2 * (P.intel - 1);
    };

    // ---- phase 1: the player's action -------------------------------------------------------
    int a = (action_in < 0 || action_in >= A_COUNT) ? A_NOOP : action_in;
    if (P.sleeping || P.resting) a = A_NOOP;
    // table / furnace within one cell of the player (crafting never moves, so this is final)
    bool near_table, near_furnace;
    {
        int b = B_INVALID;
        if (l < 9) b = wb[CX_IDX((P.py - wy0 - 1 + l / 3) * WIN_PITCH + (P.px - wx0 - 1 + l % 3), WIN_ROWS * WIN_PITCH)];
        near_table = G::ballot(b == B_TABLE) != 0;
        near_furnace = G::ballot(b == B_FURNACE) != 0;
    }
    auto try_craft = [&](bool need_furnace, int wood, int stone, int coal, int iron, int diamond) -> bool {
        if (!near_table || (need_furnace && !near_furnace)) return false;
        if (P.inv[I_WOOD] < wood || P.inv[I_STONE] < stone || P.inv[I_COAL] < coal || P.inv[I_IRON] < iron || P.inv[I_DIAMOND] < diamond) return false;
        P.inv[I_WOOD] -= wood; P.inv[I_STONE] -= stone; P.inv[I_COAL] -= coal; P.inv[I_IRON] -= iron; P.inv[I_DIAMOND] -= diamond;
        return true;
    };
    auto change_floor = [&](int nf, int x, int y) {
        const uint32_t nw = l < NSLOT ? genv[REC_DWORDS + nf * MOBTAB_DWORDS + l] : 0u;
        const Mob u = unpack_mob(nw);
        if (G::ballot(u.alive && u.x == x && u.y == y)) return;           // the far end of the ladder must be free
        if (l < NSLOT) {
            Mob o; o.alive = m.alive; o.x = m.x; o.y = m.y; o.dir = m.dir; o.hp = m.hp; o.cd = m.cd; o.type = m.type;
            genv[REC_DWORDS + P.floor * MOBTAB_DWORDS + l] = pack_mob(o);
        }
        m.alive = u.alive; m.x = u.x; m.y = u.y; m.dir = u.dir; m.hp = u.hp; m.cd = u.cd; m.type = u.type;
        P.floor = nf; P.px = x; P.py = y;
        if (!((P.visited >> nf) & 1)) {
            P.visited |= 1 << nf;
            if (P.xp < 15) ++P.xp;                                       // section "Attributes": a point per new floor
            const int ea = enter_ach(nf);
            if (ea >= 0) unlock(P, ea);
        }
        wave_sync();
        wx0 = x - WIN_COLS / 2; wy0 = y - WIN_ROWS / 2;
        load_window<GW>(l, maps, nf, x, y, wb, wi);
        wave_sync();
    };
    // a projectile of the player leaves the facing cell
    auto shoot = [&](int kind, int tx, int ty, bool t_ok) -> bool {
        if (!t_ok) return false;
        const uint32_t om = occ_mask(tx, ty);
        if (om) {
            const int k = __builtin_ctz(om);
            if (k >= S_MPROJ0) return false;
            int ap, af, ai;
            shot_attack(kind, ap, af, ai);
            hurt_mob(k, ap, af, ai);
            return true;
        }
        const uint32_t free_slots = ~(uint32_t)G::ballot(m.alive) & (7u << S_PPROJ0);
        if (!free_slots || !in_set(FLYABLE, win_b(tx, ty))) return false;
        spawn_mob(__builtin_ctz(free_slots), tx, ty, P.dir, kind, 0);
        return true;
    };

    if (a >= A_LEFT && a <= A_DOWN) {
        P.dir = a;
        const int tx = P.px + dir_dx(a), ty = P.py + dir_dy(a);
        if (inb(tx, ty) && occ_mask(tx, ty) == 0) {
            const int b = win_b(tx, ty);
            if (in_set(WALKABLE, b)) { P.px = tx; P.py = ty; }
            else if (b == B_LAVA) { P.px = tx; P.py = ty; P.vit[V_HEALTH] = 0; }
        }
    } else if (a != A_NOOP) {
        const int tx = P.px + dir_dx(P.dir), ty = P.py + dir_dy(P.dir);
        const bool t_ok = inb(tx, ty);
        const int f = P.floor;
        auto collect = [&](int b, int item, int level, int ach, int leaves) {
            if (P.pickaxe >= level && P.inv[item] < INV_MAX) {
                ++P.inv[item];
                if (leaves != b) set_facing_block(tx, ty, leaves);
                unlock(P, ach);
            }
        };
        switch (a) {
        case A_DO: {
            if (!t_ok) break;
            const uint32_t om = occ_mask(tx, ty);
            if (om) {
                const int sw = P.sword;                       // fist 1, wood 2, stone 3, iron 5, diamond 8
                const int ap = (sw == 0 ? 1 : sw == 1 ? 2 : sw == 2 ? 3 : sw == 3 ? 5 : 8) + (P.str - 1);
                hurt_mob(__builtin_ctz(om), ap, P.sword_ench == 1 ? 4 : 0, P.sword_ench == 2 ? 4 : 0);
                break;
            }
            const int b = win_b(tx, ty);
            switch (b) {
            case B_TREE: collect(b, I_WOOD, 0, H_COLLECT_WOOD, B_TREE); break;
            case B_STONE: case B_STALAGMITE: collect(b, I_STONE, 1, H_COLLECT_STONE, B_PATH); break;
            case B_COAL: collect(b, I_COAL, 1, H_COLLECT_COAL, B_PATH); break;
            case B_IRON: collect(b, I_IRON, 2, H_COLLECT_IRON, B_PATH); break;
            case B_DIAMOND: collect(b, I_DIAMOND, 3, H_COLLECT_DIAMOND, B_PATH); break;
            case B_SAPPHIRE: collect(b, I_SAPPHIRE, 4, H_COLLECT_SAPPHIRE, B_PATH); break;
            case B_RUBY: collect(b, I_RUBY, 4, H_COLLECT_RUBY, B_PATH); break;
            case B_GRASS: if (misc[9] < P_SAPLING) collect(b, I_SAPLING, 0, H_COLLECT_SAPLING, B_GRASS); break;
            case B_WATER: case B_FOUNTAIN:
                P.vit[V_DRINK] = min(cap_need(P), P.vit[V_DRINK] + 1); P.cnt[K_THIRST] = 0; unlock(P, H_COLLECT_DRINK);
                break;
            case B_RIPE:
                P.vit[V_FOOD] = min(cap_need(P), P.vit[V_FOOD] + FOOD_PLANT); P.cnt[K_HUNGER] = 0;
                set_facing_block(tx, ty, B_PLANT);
                if (q_alive && q_x == tx && q_y == ty) q_age = 0;
                unlock(P, H_EAT_PLANT);
                break;
            case B_CHEST: {
                // section "Combat": the bow lies in a chest of the first dungeon floor; books in dungeon chests
                set_facing_block(tx, ty, B_PATH);
                unlock(P, H_OPEN_CHEST);
                if (f == 1 && !P.bow) { P.bow = 1; unlock(P, H_FIND_BOW); break; }
                const int c = (int)choice(misc[10], 6);
                set_potion(P, c, min(INV_MAX, get_potion(P, c) + 1));
                const int k = (int)choice(misc[11], 4);
                if (k == 0) P.inv[I_ARROW] = min(INV_MAX, P.inv[I_ARROW] + 4);
                else if (k == 1) P.inv[I_TORCH] = min(INV_MAX, P.inv[I_TORCH] + 4);
                else if (k == 2 && P.book < 2) ++P.book;
                break;
            }
            case B_NECRO_VULN: {
                // section "Boss Floor": every hit calls the next wave; eight hits win
                unlock(P, H_DAMAGE_NECROMANCER);
                ++P.boss_hits;
                P.boss_vulnerable = 0;
                if (P.boss_hits >= BOSS_HITS) { unlock(P, H_DEFEAT_NECROMANCER); set_facing_block(tx, ty, B_PATH); break; }
                set_facing_block(tx, ty, B_NECROMANCER);
                const int wv = P.boss_hits - 1;
                const int mt = melee_of_floor(wv), rt = ranged_of_floor(wv);
#pragma unroll
                for (int s = 0; s < 5; ++s) {
                    const int x = s < 3 ? 20 + 4 * s : 22 + 4 * (s - 3), y = s < 3 ? 10 : 8;
                    const int type = s < 3 ? mt : rt;
                    const bool taken = occ_mask(x, y) != 0 || (P.px == x && P.py == y);
                    if (!G::get(m.alive, s) && !taken) spawn_mob(s, x, y, 0, type, creature(type).hp);
                }
                break;
            }
            default: break;
            }
            break;
        }
        case A_SLEEP: if (P.vit[V_ENERGY] < cap_need(P)) P.sleeping = 1; break;
        case A_REST: if (P.vit[V_HEALTH] < cap_health(P)) P.resting = 1; break;
        case A_PLACE_STONE: case A_PLACE_TABLE: case A_PLACE_FURNACE: case A_PLACE_PLANT: case A_PLACE_TORCH: {
            if (!t_ok || occ_mask(tx, ty) != 0) break;
            const int il = win_i(tx, ty);
            if ((il & 7) != IT_NONE) break;
            const int b = win_b(tx, ty);
            if (a == A_PLACE_STONE) {
                if (P.inv[I_STONE] < 1 || !in_set(FLYABLE, b)) break;
                --P.inv[I_STONE]; set_facing_block(tx, ty, B_STONE); unlock(P, H_PLACE_STONE);
            } else if (a == A_PLACE_TABLE) {
                if (P.inv[I_WOOD] < 1 || !in_set(WALKABLE, b)) break;
                --P.inv[I_WOOD]; set_facing_block(tx, ty, B_TABLE); unlock(P, H_PLACE_TABLE);
            } else if (a == A_PLACE_FURNACE) {
                if (P.inv[I_STONE] < 1 || !in_set(WALKABLE, b) || !near_table) break;
                --P.inv[I_STONE]; set_facing_block(tx, ty, B_FURNACE); unlock(P, H_PLACE_FURNACE);
            } else if (a == A_PLACE_PLANT) {
                if (f != 0 || P.inv[I_SAPLING] < 1 || b != B_GRASS) break;
                const uint32_t cap = min(p.cap_plant, (uint32_t)NPLANT);
                const uint32_t free_slots = ~(uint32_t)G::ballot(q_alive != 0) & ((1u << cap) - 1u);
                if (!free_slots) break;
                const int s = __builtin_ctz(free_slots);
                --P.inv[I_SAPLING]; set_facing_block(tx, ty, B_PLANT);
                if (l == s) { q_alive = 1; q_x = tx; q_y = ty; q_age = 0; q_block = B_PLANT; }
                unlock(P, H_PLACE_PLANT);
            } else {
                if (P.inv[I_TORCH] < 1 || !in_set(WALKABLE, b)) break;
                --P.inv[I_TORCH];
                if (l == 0) wi[CX_IDX((ty - wy0) * WIN_PITCH + (tx - wx0), WIN_ROWS * WIN_PITCH)] = (uint8_t)((il & ~7) | IT_TORCH);
                wave_sync();
                // light falls off by 4 per cell of Chebyshev distance; the centre cell also carries the item
#pragma unroll
                for (int it = 0; it < (81 + GW - 1) / GW; ++it) {
                    const int i = l + GW * it;
                    if (i < 81) {
                        const int ddy = i / 9 - 4, ddx = i % 9 - 4, x = tx + ddx, y = ty + ddy;
                        if (inb(x, y) && in_win(x, y)) {
                            const int old = wi[CX_IDX((y - wy0) * WIN_PITCH + (x - wx0), WIN_ROWS * WIN_PITCH)];
                            const int nl = MAX_LIGHT - 4 * max(iabs(ddx), iabs(ddy));
                            const bool centre = ddx == 0 && ddy == 0;
                            if (nl > (old >> 3) || centre) {
                                const int nv = (old & 7) | (max(nl, old >> 3) << 3);
                                wi[CX_IDX((y - wy0) * WIN_PITCH + (x - wx0), WIN_ROWS * WIN_PITCH)] = (uint8_t)nv;
                                maps[il_off(f, x, y)] = (uint8_t)nv;
                            }
                        }
                    }
                }
                wave_sync();
                unlock(P, H_PLACE_TORCH);
            }
            break;
        }
        // tools are levels (1 wood, 2 stone, 3 iron, 4 diamond); crafting only ever raises the level
        case A_MAKE_WOOD_PICKAXE: if (P.pickaxe < 1 && try_craft(false, 1, 0, 0, 0, 0)) { P.pickaxe = 1; unlock(P, H_MAKE_WOOD_PICKAXE); } break;
        case A_MAKE_STONE_PICKAXE: if (P.pickaxe < 2 && try_craft(false, 1, 1, 0, 0, 0)) { P.pickaxe = 2; unlock(P, H_MAKE_STONE_PICKAXE); } break;
        case A_MAKE_IRON_PICKAXE: if (P.pickaxe < 3 && try_craft(true, 1, 0, 1, 1, 0)) { P.pickaxe = 3; unlock(P, H_MAKE_IRON_PICKAXE); } break;
        case A_MAKE_DIAMOND_PICKAXE: if (P.pickaxe < 4 && try_craft(true, 1, 0, 0, 0, 3)) { P.pickaxe = 4; unlock(P, H_MAKE_DIAMOND_PICKAXE); } break;
        case A_MAKE_WOOD_SWORD: if (P.sword < 1 && try_craft(false, 1, 0, 0, 0, 0)) { P.sword = 1; unlock(P, H_MAKE_WOOD_SWORD); } break;
        case A_MAKE_STONE_SWORD: if (P.sword < 2 && try_craft(false, 1, 1, 0, 0, 0)) { P.sword = 2; unlock(P, H_MAKE_STONE_SWORD); } break;
        case A_MAKE_IRON_SWORD: if (P.sword < 3 && try_craft(true, 1, 0, 1, 1, 0)) { P.sword = 3; unlock(P, H_MAKE_IRON_SWORD); } break;
        case A_MAKE_DIAMOND_SWORD: if (P.sword < 4 && try_craft(true, 1, 0, 0, 0, 2)) { P.sword = 4; unlock(P, H_MAKE_DIAMOND_SWORD); } break;
        case A_MAKE_IRON_ARMOUR: case A_MAKE_DIAMOND_ARMOUR: {
            const int lvl = a == A_MAKE_IRON_ARMOUR ? 1 : 2;
            int piece = -1;
#pragma unroll
            for (int i = 3; i >= 0; --i) if ((int)((P.armour >> (2 * i)) & 3u) < lvl) piece = i;
            if (piece < 0) break;
            if (lvl == 1 ? try_craft(true, 0, 0, 3, 3, 0) : try_craft(true, 0, 0, 0, 0, 3)) {
                P.armour = (P.armour & ~(3u << (2 * piece))) | ((uint32_t)lvl << (2 * piece));
                unlock(P, lvl == 1 ? H_MAKE_IRON_ARMOUR : H_MAKE_DIAMOND_ARMOUR);
            }
            break;
        }
        case A_MAKE_ARROW: if (try_craft(false, 1, 1, 0, 0, 0)) { P.inv[I_ARROW] = min(INV_MAX, P.inv[I_ARROW] + 2); unlock(P, H_MAKE_ARROW); } break;
        case A_MAKE_TORCH: if (try_craft(false, 1, 0, 1, 0, 0)) { P.inv[I_TORCH] = min(INV_MAX, P.inv[I_TORCH] + 4); unlock(P, H_MAKE_TORCH); } break;
        case A_SHOOT_ARROW: if (P.bow && P.inv[I_ARROW] >= 1 && shoot(PP_ARROW, tx, ty, t_ok)) { --P.inv[I_ARROW]; unlock(P, H_FIRE_BOW); } break;
        case A_CAST_FIREBALL: if (P.fireball && P.vit[V_MANA] >= 2 && shoot(PP_FIREBALL, tx, ty, t_ok)) { P.vit[V_MANA] -= 2; unlock(P, H_CAST_FIREBALL); } break;
        case A_CAST_ICEBALL: if (P.iceball && P.vit[V_MANA] >= 2 && shoot(PP_ICEBALL, tx, ty, t_ok)) { P.vit[V_MANA] -= 2; unlock(P, H_CAST_ICEBALL); } break;
        case A_DESCEND:
            if (f < FLOORS - 1 && (win_i(P.px, P.py) & 7) == IT_LADDER_DOWN) {
                const uint32_t lw = G::uniu(rec[R_LADDER + f + 1]);
                change_floor(f + 1, lw & 0xFF, (lw >> 8) & 0xFF);
            }
            break;
        case A_ASCEND:
            if (f > 0 && (win_i(P.px, P.py) & 7) == IT_LADDER_UP) {
                const uint32_t lw = G::uniu(rec[R_LADDER + f - 1]);
                change_floor(f - 1, (lw >> 16) & 0xFF, (lw >> 24) & 0xFF);
            }
            break;
        case A_READ_BOOK:
            if (P.book < 1 || (P.fireball && P.iceball)) break;
            --P.book;
            if (!P.fireball) { P.fireball = 1; unlock(P, H_LEARN_FIREBALL); }
            else { P.iceball = 1; unlock(P, H_LEARN_ICEBALL); }
            break;
        case A_ENCHANT_SWORD: case A_ENCHANT_ARMOUR: case A_ENCHANT_BOW: {
            // section "Potions and Enchantments": mana and a gemstone at an enchantment table
            if (!t_ok) break;
            const int b = win_b(tx, ty);
            if (b != B_ENCH_FIRE && b != B_ENCH_ICE) break;
            const int elem = b == B_ENCH_FIRE ? 1 : 2;
            const int gems = elem == 1 ? P.inv[I_RUBY] : P.inv[I_SAPPHIRE];
            if (P.vit[V_MANA] < 9 || gems < 1) break;
            if (a == A_ENCHANT_SWORD) { if (P.sword < 1 || P.sword_ench == elem) break; P.sword_ench = elem; unlock(P, H_ENCHANT_SWORD); }
            else if (a == A_ENCHANT_BOW) { if (!P.bow || P.bow_ench == elem) break; P.bow_ench = elem; }
            else {
                int piece = -1;
#pragma unroll
                for (int i = 3; i >= 0; --i)
                    if (((P.armour >> (2 * i)) & 3u) > 0u && (int)((P.armour_ench >> (2 * i)) & 3u) != elem) piece = i;
                if (piece < 0) break;
                P.armour_ench = (P.armour_ench & ~(3u << (2 * piece))) | ((uint32_t)elem << (2 * piece));
                unlock(P, H_ENCHANT_ARMOUR);
            }
            P.vit[V_MANA] -= 9;
            if (elem == 1) --P.inv[I_RUBY]; else --P.inv[I_SAPPHIRE];
            break;
        }
        case A_LEVEL_UP_DEXTERITY: if (P.xp >= 1 && P.dex < 5) { --P.xp; ++P.dex; } break;
        case A_LEVEL_UP_STRENGTH: if (P.xp >= 1 && P.str < 5) { --P.xp; ++P.str; } break;
        case A_LEVEL_UP_INTELLIGENCE: if (P.xp >= 1 && P.intel < 5) { --P.xp; ++P.intel; } break;
        default:
            if (a >= A_DRINK_POTION_RED && a <= A_DRINK_POTION_YELLOW) {
                const int col = a - A_DRINK_POTION_RED, have = get_potion(P, col);
                if (have < 1) break;
                set_potion(P, col, have - 1);
                unlock(P, H_DRINK_POTION);
                // effects: health, mana or energy, +8 or -3, under this episode's colour map
                const int eff = (P.perm >> (3 * col)) & 7u, which = eff >> 1, delta = (eff & 1) ? -3 : 8;
                if (which == 0) P.vit[V_HEALTH] = max(0, min(cap_health(P), P.vit[V_HEALTH] + delta));
                else if (which == 1) P.vit[V_MANA] = max(0, min(cap_mana(P), P.vit[V_MANA] + delta));
                else P.vit[V_ENERGY] = max(0, min(cap_need(P), P.vit[V_ENERGY] + delta));
            }
            break;
        }
    }

    // ---- phase 2: mobs of the current floor ---------------------------------------------------
    const int f = P.floor;
    int damage = 0;
    {
        int pdp = 0, pdf = 0, pdi = 0;                            // the player's defence from armour
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            pdp += 10 * (int)((P.armour >> (2 * i)) & 3u);
            const int en = (P.armour_ench >> (2 * i)) & 3u;
            if (en == 1) pdf += 20;
            if (en == 2) pdi += 20;
        }
        const int idle_factor = (P.sleeping || P.resting) ? 2 : 1;

        // every live slot decides what it wants to do from the state after the player's action
        int kind = N_NONE, tx = 0, ty = 0, tdir = 0, dmg = 0, col = COL_FLYING;
        bool want_terrain = false;
        if (m.alive) {
            const int dx = P.px - m.x, dy = P.py - m.y, adx = iabs(dx), ady = iabs(dy), cheb = max(adx, ady);
            const uint32_t m8 = choice(rnd.w[0], 8);
            const int wander = m8 < 4 ? (int)m8 + 1 : 0;
            if (l < S_MPROJ0) {
                const CreatureRow c = creature(m.type);
                dmg = idle_factor * through(c.dp, c.df, c.di, pdp, pdf, pdi);
                col = c.col;
                if (l < S_RANGED0) {
                    if (m.cd > 0) --m.cd;
                    if (adx + ady == 1) { if (m.cd == 0) { kind = N_DAMAGE; m.cd = CD_MELEE; } }
                    else { tdir = (cheb < CHASE_RANGE && rnd.w[1] < P_CHASE) ? toward(dx, dy) : wander; kind = N_MOVE; }
                } else if (l < S_PASSIVE0) {
                    if (m.cd > 0) --m.cd;
                    const bool aligned = (dx == 0 || dy == 0) && cheb <= SHOOT_RANGE;
                    if (aligned && m.cd == 0 && rnd.w[1] < P_SHOOT) {
                        tdir = toward(dx, dy);
                        m.cd = CD_RANGED;
                        kind = (m.x + dir_dx(tdir) == P.px && m.y + dir_dy(tdir) == P.py) ? N_DAMAGE : N_SHOOT;
                        col = COL_FLYING;
                    } else { tdir = wander ? wander : (cheb <= SHOOT_RANGE ? toward(dx, dy) : 0); kind = N_MOVE; }
                } else { tdir = wander; kind = N_MOVE; }
                if (tdir == 0 && kind == N_MOVE) kind = N_NONE;
            } else {
                tdir = m.dir;
                if (l < S_PPROJ0) {
                    const CreatureRow c = creature(m.type);
                    dmg = idle_factor * through(c.dp, c.df, c.di, pdp, pdf, pdi);
                    kind = N_FLY;
                } else kind = N_PPROJ;
            }
            tx = m.x + dir_dx(tdir); ty = m.y + dir_dy(tdir);
            const bool at_player = tx == P.px && ty == P.py;
            if (kind == N_FLY && at_player) kind = N_DAMAGE_DIE;
            if (kind == N_MOVE || kind == N_SHOOT || kind == N_FLY || kind == N_PPROJ) {
                if (!inb(tx, ty)) kind = (kind == N_FLY || kind == N_PPROJ) ? N_DIE : N_NONE;
                else want_terrain = true;
            }
        }
        // spawn candidates of the three classes (lanes 0..2 fetch their terrain with the mobs)
        int sx[3], sy[3];
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            sx[j] = P.px + (int)choice(misc[3 * j], 31) - 15;
            sy[j] = P.py + (int)choice(misc[3 * j + 1], 31) - 15;
        }
        int probe_b = B_INVALID;
        {
            const int x = l == 0 ? sx[0] : (l == 1 ? sx[1] : sx[2]), y = l == 0 ? sy[0] : (l == 1 ? sy[1] : sy[2]);
            if (l < 3 && f != 8 && inb(x, y)) {
                probe_b = maps[block_off(f, x, y)];
                if (patch_f == f && patch_x == x && patch_y == y) probe_b = patch_b;
            }
        }
        bool ok = false;
        if (want_terrain) {
            int b = maps[block_off(f, tx, ty)];
            if (patch_f == f && patch_x == tx && patch_y == ty) b = patch_b;
            ok = passable_for(col, b);
            if (kind == N_FLY && !ok) kind = N_DIE;
            if (kind == N_PPROJ && tx == P.px && ty == P.py) ok = false;
        }
        const int iwv = kind | ((tx & 63) << 4) | ((ty & 63) << 10) | ((ok ? 1 : 0) << 16) | (dmg << 17) | (tdir << 25);

        // the slots act one after the other, each seeing what the earlier ones did
        uint32_t alive_bits = (uint32_t)G::ballot(m.alive != 0);
        constexpr int ORDER[NSLOT] = { 0, 1, 2, 5, 6, 7, 8, 9, 10, 11, 12, 13, 3, 4 };
#pragma unroll
        for (int i = 0; i < NSLOT; ++i) {
            const int k = ORDER[i];
            if (!((alive_bits >> k) & 1u)) continue;
            const int iw = G::get(iwv, k);
            const int kd = iw & 15, kx = (iw >> 4) & 63, ky = (iw >> 10) & 63, kdir = (iw >> 25) & 7;
            const bool kok = (iw >> 16) & 1;
            const int kdmg = (iw >> 17) & 255;
            if (kd == N_NONE) continue;
            if (kd == N_DAMAGE) { damage += kdmg; continue; }
            if (kd == N_DAMAGE_DIE || kd == N_DIE) {
                if (kd == N_DAMAGE_DIE) damage += kdmg;
                if (l == k) clear_mob(m);
                alive_bits &= ~(1u << k);
                continue;
            }
            const uint32_t om = occ_mask(kx, ky);
            if (kd == N_MOVE) {
                if (kok && om == 0 && !(kx == P.px && ky == P.py) && l == k) { m.x = kx; m.y = ky; }
            } else if (kd == N_SHOOT) {
                const uint32_t free_slots = ~alive_bits & (7u << S_MPROJ0);
                if (free_slots && kok && om == 0) {
                    const int s = __builtin_ctz(free_slots);
                    const int type = G::get(m.type, k);
                    if (l == s) { m.alive = 1; m.x = kx; m.y = ky; m.dir = kdir; m.hp = 0; m.cd = 0; m.type = type; }
                    alive_bits |= 1u << s;
                }
            } else if (kd == N_FLY) {
                if (om) { if (l == k) clear_mob(m); alive_bits &= ~(1u << k); }
                else if (l == k) { m.x = kx; m.y = ky; }
            } else {   // N_PPROJ
                if (om) {
                    const int hit = __builtin_ctz(om);
                    int ap, af, ai;
                    shot_attack(G::get(m.type, k), ap, af, ai);
                    if (hurt_mob(hit, ap, af, ai)) alive_bits &= ~(1u << hit);
                    if (l == k) clear_mob(m);
                    alive_bits &= ~(1u << k);
                } else if (kok) { if (l == k) { m.x = kx; m.y = ky; } }
                else { if (l == k) clear_mob(m); alive_bits &= ~(1u << k); }
            }
        }
        P.vit[V_HEALTH] = max(0, P.vit[V_HEALTH] - damage);

        // ---- despawn far away, spawn near (section "Creatures": fixed slots, masked when empty) ----
        if (m.alive && max(iabs(m.x - P.px), iabs(m.y - P.py)) > DESPAWN_DIST) clear_mob(m);
        alive_bits = (uint32_t)G::ballot(m.alive != 0);
        if (f == 8) {
            // the necromancer can be hit again once its wave is gone
            if (!P.boss_vulnerable && P.boss_hits < BOSS_HITS && !(alive_bits & 0x1Fu)) {
                P.boss_vulnerable = 1;
                set_block(BOSS_X, BOSS_Y, B_NECRO_VULN);
            }
        } else {
            const int first[3] = { S_MELEE0, S_RANGED0, S_PASSIVE0 }, count[3] = { 3, 2, 3 };
            const uint32_t caps[3] = { p.cap_melee, p.cap_ranged, p.cap_passive };
            const int type[3] = { melee_of_floor(f), ranged_of_floor(f), passive_of_floor(f) };
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const int x = sx[j], y = sy[j];
                const int n = min(count[j], (int)caps[j]);
                const uint32_t free_slots = ~alive_bits & (((1u << n) - 1u) << first[j]);
                if (type[j] < 0 || !free_slots || max(iabs(x - P.px), iabs(y - P.py)) < SPAWN_MIN_DIST || !inb(x, y)) continue;
                if (occ_mask(x, y) != 0 || (x == P.px && y == P.py)) continue;
                const int b = G::get(probe_b, j);
                uint32_t thr; bool okb;
                if (f == 0) {   // overworld: zombies on grass by darkness, skeletons on paths, cows on grass
                    thr = j == 0 ? zombie_thr : (j == 1 ? P_SKELETON_SPAWN : P_PASSIVE_SPAWN);
                    okb = j == 1 ? b == B_PATH : b == B_GRASS;
                } else {
                    thr = j == 0 ? P_MELEE_SPAWN : (j == 1 ? P_RANGED_SPAWN : P_PASSIVE_SPAWN);
                    okb = passable_for(creature(type[j]).col, b);
                }
                if (!okb || misc[3 * j + 2] >= thr) continue;
                const int s = __builtin_ctz(free_slots);
                spawn_mob(s, x, y, 0, type[j], creature(type[j]).hp);
                alive_bits |= 1u << s;
            }
        }
    }

    // ---- plants: they only grow while the player is in the overworld ---------------------------
    if (f == 0) {
        if (patch_f == 0 && patch_x == q_x && patch_y == q_y) q_block = patch_b;
        const int z0 = G::get(m.alive, 0) ? (G::get(m.x, 0) | (G::get(m.y, 0) << 8)) : -1;
        const int z1 = G::get(m.alive, 1) ? (G::get(m.x, 1) | (G::get(m.y, 1) << 8)) : -1;
        const int z2 = G::get(m.alive, 2) ? (G::get(m.x, 2) | (G::get(m.y, 2) << 8)) : -1;
        if (l < NPLANT && q_alive) {
            if (q_age < 65535) ++q_age;
            const int x = q_x, y = q_y;
            int nb = -1;
            if (q_block == B_PLANT && q_age >= RIPE_AGE) nb = B_RIPE;
            auto beside = [&](int z) { return z >= 0 && iabs((z & 0xFF) - q_x) + iabs((z >> 8) - q_y) == 1; };
            if ((beside(z0) || beside(z1) || beside(z2)) && rnd.w[2] < P_PLANT_EATEN) { nb = B_GRASS; q_alive = 0; q_x = q_y = q_age = 0; }
            if (nb >= 0) {
                maps[block_off(0, x, y)] = (uint8_t)nb;
                if (in_win(x, y)) wb[CX_IDX((y - wy0) * WIN_PITCH + (x - wx0), WIN_ROWS * WIN_PITCH)] = (uint8_t)nb;
            }
        }
        wave_sync();
    }
    qw = q_alive ? (1u | ((uint32_t)q_x << 1) | ((uint32_t)q_y << 7) | ((uint32_t)q_age << 16)) : 0u;

    // ---- needs -------------------------------------------------------------------------------
    {
        const bool damaged = damage > 0;
        const int asleep = P.sleeping, idle = P.sleeping || P.resting;
        P.cnt[K_HUNGER] += asleep ? 1 : 2;
        if (P.cnt[K_HUNGER] > 50) { P.cnt[K_HUNGER] = 0; P.vit[V_FOOD] = max(0, P.vit[V_FOOD] - 1); }
        P.cnt[K_THIRST] += asleep ? 1 : 2;
        if (P.cnt[K_THIRST] > 40) { P.cnt[K_THIRST] = 0; P.vit[V_DRINK] = max(0, P.vit[V_DRINK] - 1); }
        if (asleep) {
            --P.cnt[K_FATIGUE];
            if (P.cnt[K_FATIGUE] < -10) { P.cnt[K_FATIGUE] = 0; P.vit[V_ENERGY] = min(cap_need(P), P.vit[V_ENERGY] + 1); }
        } else {
            ++P.cnt[K_FATIGUE];
            if (P.cnt[K_FATIGUE] > 30) { P.cnt[K_FATIGUE] = 0; P.vit[V_ENERGY] = max(0, P.vit[V_ENERGY] - 1); }
        }
        P.cnt[K_MANA] += P.intel;                             // section "Attributes": intelligence feeds magic
        if (P.cnt[K_MANA] > 20) { P.cnt[K_MANA] = 0; P.vit[V_MANA] = min(cap_mana(P), P.vit[V_MANA] + 1); }
        if (P.vit[V_HEALTH] > 0) {
            const bool fed = P.vit[V_FOOD] > 0 && P.vit[V_DRINK] > 0 && (P.vit[V_ENERGY] > 0 || asleep);
            P.cnt[K_RECOVER] += fed ? (idle ? 4 : 2) : (idle ? -1 : -2);
            if (P.cnt[K_RECOVER] > 50) { P.cnt[K_RECOVER] = 0; P.vit[V_HEALTH] = min(cap_health(P), P.vit[V_HEALTH] + 1); }
            if (P.cnt[K_RECOVER] < -30) { P.cnt[K_RECOVER] = 0; --P.vit[V_HEALTH]; }
        }
        if (asleep && (P.vit[V_ENERGY] >= cap_need(P) || damaged)) { P.sleeping = 0; unlock(P, H_WAKE_UP); }
        if (P.resting && (P.vit[V_HEALTH] >= cap_health(P) || damaged)) P.resting = 0;
    }

    // ---- reward, time, done (section "RL Environment Interface") ------------------------------
    int gained = 0;
    StepOut o;
#pragma unroll
    for (int w = 0; w < 3; ++w) {
        const uint32_t nw = P.ach[w] & ~ach0[w];
        o.unlocked[w] = nw;
        gained += __builtin_popcount(nw & CAT1[w]) + 3 * __builtin_popcount(nw & CAT3[w]) +
                  5 * __builtin_popcount(nw & CAT5[w]) + 8 * __builtin_popcount(nw & CAT8[w]);
    }
    o.reward = (float)(10 * gained + (P.vit[V_HEALTH] - health0)) * 0.1f;
    ++P.t;
    P.phase = P.phase + 1 == (int)p.day_length ? 0 : P.phase + 1;
    o.done = P.vit[V_HEALTH] <= 0 || P.t >= p.max_episode_steps;
    o.wx0 = wx0; o.wy0 = wy0;
    return o;
}

}  // namespace cf
