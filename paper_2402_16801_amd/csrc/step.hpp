// One Craftax-Classic step of one environment, executed by the 16 lanes that own it.
//
// What the paper fixes: 17 actions that are always legal and fall back to a no-op when their
// prerequisites are missing (section "RL Environment Interface"), 22 achievements worth +1
// the first time and +-0.1 per health point (same section), fixed-capacity creature and plant
// tables whose empty slots are masked (appendix "Differences between Craftax-Classic and
// Crafter"), creature health and damage (appendix "Creatures").  The remaining rules
// ("mimic Crafter") are this library's own frozen reading.
//
// Lane roles: every lane carries the player's state redundantly (same inputs, same
// arithmetic, so no exchange is needed); lane k < 12 owns mob slot k, lane k < 10 owns plant
// slot k, lane k < 12 evaluates Philox block k of the step.  Random draws have fixed slots:
// block k = (move draw of mob k, decision draw of mob k, eaten draw of plant k, misc[k]);
// misc[3j..3j+2] = (x, y, p) of the spawn attempt of type j; misc[9] = sapling draw.
#pragma once

#include "common.hpp"

namespace cx {

enum Intent : int { K_NONE = 0, K_MOVE = 1, K_MOVE_PATH = 2, K_ATTACK = 3, K_SHOOT = 4, K_FLY = 5 };

struct StepOut { bool done; float reward; };

// Returns with the record in LDS (*r) updated unless the episode ended.
__device__ inline StepOut step_env(int l, uint32_t env, EnvRec* r, uint8_t* __restrict__ map,
                                   const Luts* __restrict__ luts, int action, const Params& p)
{
    // ---- unpack -----------------------------------------------------------------------------
    int px = r->px, py = r->py, dir = r->dir, sleeping = r->sleeping;
    int inv[12], vit[4], cnt[4];
#pragma unroll
    for (int i = 0; i < 12; ++i) inv[i] = r->inv[i];
#pragma unroll
    for (int i = 0; i < 4; ++i) { vit[i] = r->vit[i]; cnt[i] = r->cnt[i]; }
    uint32_t ach = r->ach;
    const uint32_t t = r->t, episode = r->episode, seed_lo = r->seed_lo, seed_hi = r->seed_hi;
    uint32_t phase = r->phase;
    int m_alive = 0, m_x = 0, m_y = 0, m_dir = 0, m_hp = 0, m_cd = 0;
    if (l < NMOB) {
        const Mob m = r->mob[l];
        m_alive = m.alive; m_x = m.x; m_y = m.y; m_dir = m.dir; m_hp = m.hp; m_cd = m.cd;
    }
    int p_alive = 0, p_x = 0, p_y = 0, p_age = 0;
    if (l < NPLANT) {
        const Plant q = r->plant[l];
        p_alive = q.alive; p_x = q.x; p_y = q.y; p_age = q.age;
    }
    const int health0 = vit[0];
    const uint32_t ach0 = ach;

    const U4 dr = philox4x32_10(env, t, episode, (DOM_STEP << 16) | (uint32_t)l, seed_lo, seed_hi);
    const uint32_t sapling_draw = (uint32_t)gshfl((int)dr.w[3], 9);

    int a = ((unsigned)action < (unsigned)AC_COUNT) ? action : (int)AC_NOOP;
    if (sleeping) a = AC_NOOP;

    // ---- the 3x3 neighbourhood of the player: lane j < 9 holds cell (px-1+j%3, py-1+j/3) ---
    int nb = BK_OOB;
    if (l < 9) {
        const int x = px - 1 + l % 3, y = py - 1 + l / 3;
        if (in_map(x, y)) nb = map[y * MAPW + x];
    }
    // plant cells are read now as well; the value is patched below if this step's action edits it
    int p_block = BK_INVALID;
    if (l < NPLANT && p_alive) p_block = map[p_y * MAPW + p_x];

    const bool near_table = gballot(l < 9 && nb == BK_TABLE) != 0;
    const bool near_furnace = gballot(l < 9 && nb == BK_FURNACE) != 0;

    // ---- phase 1: the player's action ----------------------------------------------------------
    if (a >= AC_LEFT && a <= AC_DOWN) dir = a;
    const int ddx = dir_dx(dir), ddy = dir_dy(dir);
    const int fx = px + ddx, fy = py + ddy;
    const bool f_in = in_map(fx, fy);
    const int fb = gshfl(nb, (ddy + 1) * 3 + (ddx + 1));
    const uint32_t hitmask = gballot(l < NMOB && m_alive && m_x == fx && m_y == fy);
    const int hit = hitmask ? (__ffs((int)hitmask) - 1) : -1;
    const int hit_hp = gshfl(m_hp, hit < 0 ? 0 : hit);
    const uint32_t plant_mask = gballot(l < NPLANT && p_alive);

    int modcell = -1, modval = 0;    // the single map cell the action may change
    bool plant_new = false, plant_eaten_by_player = false;

    if (a >= AC_LEFT && a <= AC_DOWN) {
        if (f_in && hit < 0) {
            if (walkable_ground(fb)) { px = fx; py = fy; }
            else if (fb == BK_LAVA) { px = fx; py = fy; vit[0] = 0; }
        }
    } else if (a == AC_DO) {
        if (f_in) {
            if (hit >= 0) {
                const int type = hit / 3;
                if (type != MT_ARROW) {
                    const int dmg = inv[IV_IRON_SWORD] ? 5 : (inv[IV_STONE_SWORD] ? 3 : (inv[IV_WOOD_SWORD] ? 2 : 1));
                    const int hp = hit_hp - dmg;
                    if (hp > 0) {
                        if (l == hit) m_hp = hp;
                    } else {
                        if (l == hit) { m_alive = 0; m_x = 0; m_y = 0; m_dir = 0; m_hp = 0; m_cd = 0; }
                        if (type == MT_ZOMBIE) ach |= 1u << ACH_DEFEAT_ZOMBIE;
                        if (type == MT_SKELETON) ach |= 1u << ACH_DEFEAT_SKELETON;
                        if (type == MT_COW) {
                            vit[1] = min(MAX_COUNT, vit[1] + FOOD_COW);
                            cnt[0] = 0;
                            ach |= 1u << ACH_EAT_COW;
                        }
                    }
                }
            } else {
                int item = -1, leaves = fb, achv = 0;
                bool gate = true;
                switch (fb) {
                case BK_TREE: item = IV_WOOD; achv = ACH_COLLECT_WOOD; break;
                case BK_STONE: item = IV_STONE; gate = inv[IV_WOOD_PICKAXE]; leaves = BK_PATH; achv = ACH_COLLECT_STONE; break;
                case BK_COAL: item = IV_COAL; gate = inv[IV_WOOD_PICKAXE]; leaves = BK_PATH; achv = ACH_COLLECT_COAL; break;
                case BK_IRON: item = IV_IRON; gate = inv[IV_STONE_PICKAXE]; leaves = BK_PATH; achv = ACH_COLLECT_IRON; break;
                case BK_DIAMOND: item = IV_DIAMOND; gate = inv[IV_IRON_PICKAXE]; leaves = BK_PATH; achv = ACH_COLLECT_DIAMOND; break;
                case BK_GRASS: item = IV_SAPLING; gate = sapling_draw < P_SAPLING; achv = ACH_COLLECT_SAPLING; break;
                case BK_WATER:
                    vit[2] = min(MAX_COUNT, vit[2] + 1); cnt[1] = 0; ach |= 1u << ACH_COLLECT_DRINK;
                    break;
                case BK_RIPE:
                    vit[1] = min(MAX_COUNT, vit[1] + FOOD_PLANT); cnt[0] = 0; ach |= 1u << ACH_EAT_PLANT;
                    modcell = fy * MAPW + fx; modval = BK_PLANT;
                    plant_eaten_by_player = true;
                    break;
                default: break;
                }
                if (item >= 0 && gate) {
                    // inv[] is indexed with a run-time value only here; go through the items one by one
#pragma unroll
                    for (int i = 0; i < 6; ++i)
                        if (i == item && inv[i] < MAX_COUNT) {
                            inv[i]++;
                            ach |= 1u << achv;
                            if (leaves != fb) { modcell = fy * MAPW + fx; modval = leaves; }
                        }
                }
            }
        }
    } else if (a == AC_SLEEP) {
        if (vit[3] < MAX_COUNT) sleeping = 1;
    } else if (a >= AC_PLACE_STONE && a <= AC_PLACE_PLANT) {
        if (f_in && hit < 0) {
            if (a == AC_PLACE_STONE) {
                if (inv[IV_STONE] >= 1 && (walkable_ground(fb) || fb == BK_WATER || fb == BK_LAVA)) {
                    inv[IV_STONE]--; modcell = fy * MAPW + fx; modval = BK_STONE; ach |= 1u << ACH_PLACE_STONE;
                }
            } else if (a == AC_PLACE_TABLE) {
                if (inv[IV_WOOD] >= 1 && walkable_ground(fb)) {
                    inv[IV_WOOD]--; modcell = fy * MAPW + fx; modval = BK_TABLE; ach |= 1u << ACH_PLACE_TABLE;
                }
            } else if (a == AC_PLACE_FURNACE) {
                if (inv[IV_STONE] >= 1 && walkable_ground(fb) && near_table) {
                    inv[IV_STONE]--; modcell = fy * MAPW + fx; modval = BK_FURNACE; ach |= 1u << ACH_PLACE_FURNACE;
                }
            } else {
                const uint32_t free_slots = ~plant_mask & ((1u << p.cap_plant) - 1u);
                if (inv[IV_SAPLING] >= 1 && fb == BK_GRASS && free_slots) {
                    inv[IV_SAPLING]--; modcell = fy * MAPW + fx; modval = BK_PLANT; ach |= 1u << ACH_PLACE_PLANT;
                    plant_new = true;
                    if (l == __ffs((int)free_slots) - 1) { p_alive = 1; p_x = fx; p_y = fy; p_age = 0; p_block = BK_PLANT; }
                }
            }
        }
    } else if (a >= AC_MAKE_WOOD_PICKAXE) {
        // recipe table: wood, stone, coal, iron, needs furnace
        const int tier = (a - AC_MAKE_WOOD_PICKAXE) % 3;          // 0 wood, 1 stone, 2 iron
        const int item = IV_WOOD_PICKAXE + (a - AC_MAKE_WOOD_PICKAXE);
        const int need_stone = tier == 1, need_ci = tier == 2;
        int have = 0;
#pragma unroll
        for (int i = 6; i < 12; ++i) if (i == item) have = inv[i];
        const bool ok = !have && near_table && (!need_ci || near_furnace) && inv[IV_WOOD] >= 1 &&
                        inv[IV_STONE] >= need_stone && inv[IV_COAL] >= need_ci && inv[IV_IRON] >= need_ci;
        if (ok) {
            inv[IV_WOOD]--; inv[IV_STONE] -= need_stone; inv[IV_COAL] -= need_ci; inv[IV_IRON] -= need_ci;
#pragma unroll
            for (int i = 6; i < 12; ++i) if (i == item) inv[i] = 1;
            const int achs[6] = { ACH_MAKE_WOOD_PICKAXE, ACH_MAKE_STONE_PICKAXE, ACH_MAKE_IRON_PICKAXE,
                                  ACH_MAKE_WOOD_SWORD, ACH_MAKE_STONE_SWORD, ACH_MAKE_IRON_SWORD };
#pragma unroll
            for (int i = 0; i < 6; ++i) if (i == a - AC_MAKE_WOOD_PICKAXE) ach |= 1u << achs[i];
        }
    }
    if (plant_eaten_by_player && l < NPLANT && p_alive && p_x == fx && p_y == fy) { p_age = 0; }
    if (modcell >= 0) {
        if (l == 0) map[modcell] = (uint8_t)modval;
        if (l < NPLANT && p_alive && p_y * MAPW + p_x == modcell) p_block = modval;
    }
    (void)plant_new;

    // ---- phase 2: mobs.  Intent of each slot from its own state, the player and its draws ----
    int kind = K_NONE, ndir = 0;
    if (l < NMOB && m_alive) {
        const int type = l / 3;
        const int dx = px - m_x, dy = py - m_y;
        const int adx = iabs(dx), ady = iabs(dy), cheb = max(adx, ady);
        const uint32_t m8 = choice(dr.w[0], 8);
        const uint32_t r_act = dr.w[1];
        const int toward = adx >= ady ? (dx < 0 ? 1 : 2) : (dy < 0 ? 3 : 4);
        if (type == MT_ZOMBIE) {
            if (m_cd > 0) m_cd--;
            if (adx + ady == 1) {
                if (m_cd == 0) { kind = K_ATTACK; m_cd = CD_ZOMBIE; }
            } else {
                if (cheb < CHASE_RANGE && r_act < P_CHASE) ndir = toward;
                else if (m8 < 4) ndir = (int)m8 + 1;
                if (ndir) kind = K_MOVE;
            }
        } else if (type == MT_COW) {
            if (m8 < 4) { ndir = (int)m8 + 1; kind = K_MOVE; }
        } else if (type == MT_SKELETON) {
            if (m_cd > 0) m_cd--;
            const bool aligned = (dx == 0 || dy == 0) && cheb <= SHOOT_RANGE;
            if (aligned && m_cd == 0 && r_act < P_SHOOT) { kind = K_SHOOT; ndir = toward; m_cd = CD_SKELETON; }
            else {
                if (m8 < 4) ndir = (int)m8 + 1;
                else if (cheb <= SHOOT_RANGE) ndir = toward;
                if (ndir) kind = K_MOVE_PATH;
            }
        } else {
            kind = K_FLY; ndir = m_dir;
        }
    }
    const int tx = m_x + dir_dx(ndir), ty = m_y + dir_dy(ndir);
    const bool t_in = in_map(tx, ty);
    int tb = BK_OOB;
    if (kind != K_NONE && kind != K_ATTACK && t_in) {
        tb = map[ty * MAPW + tx];
        if (ty * MAPW + tx == modcell) tb = modval;
    }
    const bool at_player = (tx == px && ty == py);
    const bool t_ok = t_in && (kind == K_MOVE ? walkable_ground(tb) : (kind == K_MOVE_PATH ? tb == BK_PATH : arrow_flyable(tb)));

    // spawn candidates (phase 3) are fixed by the draws and the player's position: read their
    // terrain now so the loads overlap the mob resolution below
    int sp_x[3], sp_y[3], sp_b[3];
    bool sp_cand[3];
    uint32_t sp_p[3];
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        const int dx = (int)choice((uint32_t)gshfl((int)dr.w[3], 3 * j), 31) - 15;
        const int dy = (int)choice((uint32_t)gshfl((int)dr.w[3], 3 * j + 1), 31) - 15;
        sp_p[j] = (uint32_t)gshfl((int)dr.w[3], 3 * j + 2);
        sp_x[j] = px + dx; sp_y[j] = py + dy;
        sp_cand[j] = max(iabs(dx), iabs(dy)) >= SPAWN_MIN_DIST && in_map(sp_x[j], sp_y[j]);
        sp_b[j] = sp_cand[j] ? (int)map[sp_y[j] * MAPW + sp_x[j]] : (int)BK_OOB;
    }

    // damage does not depend on who moves where
    const int n_attack = __popc(gballot(kind == K_ATTACK));
    const int n_arrow = __popc(gballot((kind == K_SHOOT || kind == K_FLY) && at_player));
    const int damage = n_attack * (sleeping ? DMG_ZOMBIE_SLEEP : DMG_ZOMBIE) + n_arrow * DMG_ARROW;

    // Moves resolve one slot at a time in the order zombies, cows, arrows, skeletons; each sees
    // the positions left by the slots before it.  An arrow shot now first flies next step.
    const int packed = kind | ((int)t_ok << 3) | ((int)at_player << 4) | ((tx + 1) << 8) | ((ty + 1) << 16) | (ndir << 24);
    constexpr int ORDER[NMOB] = { 0, 1, 2, 3, 4, 5, 9, 10, 11, 6, 7, 8 };
#pragma unroll
    for (int i = 0; i < NMOB; ++i) {
        const int k = ORDER[i];
        const int ik = gshfl(packed, k);
        const int kk = ik & 7;
        const bool k_ok = (ik >> 3) & 1, k_at = (ik >> 4) & 1;
        const int kx = ((ik >> 8) & 0xFF) - 1, ky = ((ik >> 16) & 0xFF) - 1;
        const uint32_t alive_mask = gballot(l < NMOB && m_alive);
        const bool occ = gballot(l < NMOB && m_alive && m_x == kx && m_y == ky) != 0 || (kx == px && ky == py);
        if (kk == K_MOVE || kk == K_MOVE_PATH) {
            if (k_ok && !occ && l == k) { m_x = kx; m_y = ky; }
        } else if (kk == K_SHOOT) {
            const uint32_t free_arrows = ~(alive_mask >> 9) & ((1u << p.cap_arrow) - 1u) & 7u;
            if (!k_at && free_arrows && k_ok && !occ && l == 9 + __ffs((int)free_arrows) - 1) {
                m_alive = 1; m_x = kx; m_y = ky; m_dir = (ik >> 24) & 7; m_hp = 0; m_cd = 0;
            }
        } else if (kk == K_FLY) {
            if (l == k) {
                if (k_at || !k_ok || occ) { m_alive = 0; m_x = 0; m_y = 0; m_dir = 0; m_hp = 0; m_cd = 0; }
                else { m_x = kx; m_y = ky; }
            }
        }
    }
    vit[0] = max(0, vit[0] - damage);

    // ---- phase 3: despawn far mobs, then one spawn attempt per type -----------------------------
    if (l < NMOB && m_alive && max(iabs(m_x - px), iabs(m_y - py)) > DESPAWN_DIST) {
        m_alive = 0; m_x = 0; m_y = 0; m_dir = 0; m_hp = 0; m_cd = 0;
    }
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        const uint32_t alive_mask = gballot(l < NMOB && m_alive);
        const bool occ = gballot(l < NMOB && m_alive && m_x == sp_x[j] && m_y == sp_y[j]) != 0;
        const uint32_t cap = j == 0 ? p.cap_zombie : (j == 1 ? p.cap_cow : p.cap_skeleton);
        const uint32_t free_slots = ~(alive_mask >> (3 * j)) & ((1u << cap) - 1u) & 7u;
        const uint32_t thr = j == 0 ? luts->zombie_thr[phase] : (j == 1 ? P_COW_SPAWN : P_SKELETON_SPAWN);
        const int want = j == 2 ? BK_PATH : BK_GRASS;
        if (sp_cand[j] && free_slots && !occ && sp_b[j] == want && sp_p[j] < thr &&
            l == 3 * j + __ffs((int)free_slots) - 1) {
            m_alive = 1; m_x = sp_x[j]; m_y = sp_y[j]; m_dir = 0;
            m_hp = j == 0 ? HP_ZOMBIE : (j == 1 ? HP_COW : HP_SKELETON); m_cd = 0;
        }
    }

    // ---- phase 4: plants ----------------------------------------------------------------------------
    {
        bool zombie_near = false;
        const int me = (m_alive ? 1 : 0) | (m_x << 8) | (m_y << 16);
#pragma unroll
        for (int z = 0; z < 3; ++z) {
            const int zi = gshfl(me, z);
            const int zx = (zi >> 8) & 0xFF, zy = (zi >> 16) & 0xFF;
            zombie_near = zombie_near || ((zi & 1) && iabs(zx - p_x) + iabs(zy - p_y) == 1);
        }
        if (l < NPLANT && p_alive) {
            if (p_age < 65535) p_age++;
            int nb2 = p_block;
            if (p_block == BK_PLANT && p_age >= RIPE_AGE) nb2 = BK_RIPE;
            if (zombie_near && dr.w[2] < P_PLANT_EATEN) nb2 = BK_GRASS;
            if (nb2 != p_block) map[p_y * MAPW + p_x] = (uint8_t)nb2;
            if (nb2 == BK_GRASS) { p_alive = 0; p_x = 0; p_y = 0; p_age = 0; }
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
    const int gained = __popc(ach & ~ach0);
    out.reward = (float)(10 * gained + (vit[0] - health0)) * 0.1f;
    const uint32_t t1 = t + 1;
    phase = phase + 1 == p.day_length ? 0u : phase + 1;
    out.done = vit[0] <= 0 || t1 >= p.max_episode_steps;
    if (out.done) return out;

    // ---- pack the record back into LDS ------------------------------------------------------------------
    group_sync();
    if (l == 0) {
        uint32_t* w = reinterpret_cast<uint32_t*>(r);
        w[0] = (uint32_t)px | ((uint32_t)py << 8) | ((uint32_t)dir << 16) | ((uint32_t)sleeping << 24);
        w[1] = (uint32_t)inv[0] | ((uint32_t)inv[1] << 8) | ((uint32_t)inv[2] << 16) | ((uint32_t)inv[3] << 24);
        w[2] = (uint32_t)inv[4] | ((uint32_t)inv[5] << 8) | ((uint32_t)inv[6] << 16) | ((uint32_t)inv[7] << 24);
        w[3] = (uint32_t)inv[8] | ((uint32_t)inv[9] << 8) | ((uint32_t)inv[10] << 16) | ((uint32_t)inv[11] << 24);
        w[4] = (uint32_t)(vit[0] & 0xFF) | ((uint32_t)(vit[1] & 0xFF) << 8) | ((uint32_t)(vit[2] & 0xFF) << 16) | ((uint32_t)(vit[3] & 0xFF) << 24);
        w[5] = (uint32_t)(cnt[0] & 0xFFFF) | ((uint32_t)(cnt[1] & 0xFFFF) << 16);
        w[6] = (uint32_t)(cnt[2] & 0xFFFF) | ((uint32_t)(cnt[3] & 0xFFFF) << 16);
        w[7] = ach;
        w[8] = t1;
        w[12] = phase;
    }
    if (l < NMOB) {
        uint32_t* w = reinterpret_cast<uint32_t*>(&r->mob[l]);
        w[0] = (uint32_t)m_alive | ((uint32_t)m_x << 8) | ((uint32_t)m_y << 16) | ((uint32_t)m_dir << 24);
        w[1] = (uint32_t)(m_hp & 0xFF) | ((uint32_t)m_cd << 8);
    }
    if (l < NPLANT) {
        uint32_t* w = reinterpret_cast<uint32_t*>(&r->plant[l]);
        w[0] = (uint32_t)p_alive | ((uint32_t)p_x << 8) | ((uint32_t)p_y << 16);
        w[1] = (uint32_t)p_age;
    }
    group_sync();
    return out;
}

}  // namespace cx
