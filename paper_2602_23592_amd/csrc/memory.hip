// Static-dynamic memory construction (Section 4.1): host-side bookkeeping of segments, groups,
// their static / dynamic state over a window of steps, and of which cache units are stale.
// No device code: the file is built with the rest of the library so that one shared object
// carries the whole C ABI.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <map>
#include <set>
#include <string>
#include <vector>

#include "keep_memory.h"

namespace {

struct Segment {
  int32_t group;
  std::vector<int32_t> tokens;
  int64_t last_change;  // step during which the content was last written
  bool cached;          // its individual cache exists and matches the content
};

struct Group {
  int32_t kind = KEEP_UNIT_DYNAMIC_SEGMENT;  // dynamic groups are cached per segment
  std::set<int32_t> segments;
  int64_t last_member_change = 0;
  bool cached = false;  // the joint cache exists and matches (static groups)
};

struct UnitRef {
  int32_t kind, id, group;
};

}  // namespace

struct keep_memory {
  int32_t t = 0;
  int64_t now = 0;  // index of the open step
  std::map<int32_t, Segment> seg;
  std::map<int32_t, Group> grp;
  std::vector<UnitRef> units;  // rebuilt after every change
  bool units_valid = false;
  std::string err;
};

namespace {

keep_status mfail(keep_memory* m, keep_status st, const char* fmt, ...) {
  char buf[256];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (m) m->err = buf;
  return st;
}

void rebuild_units(keep_memory* m) {
  m->units.clear();
  for (const auto& g : m->grp) {
    if (g.second.kind == KEEP_UNIT_STATIC_GROUP) {
      m->units.push_back({KEEP_UNIT_STATIC_GROUP, g.first, g.first});
    } else {
      for (int32_t s : g.second.segments) m->units.push_back({KEEP_UNIT_DYNAMIC_SEGMENT, s, g.first});
    }
  }
  m->units_valid = true;
}

const std::vector<UnitRef>& units_of(const keep_memory* m) {
  if (!m->units_valid) rebuild_units(const_cast<keep_memory*>(m));
  return m->units;
}

bool unit_dirty(const keep_memory* m, const UnitRef& u) {
  return u.kind == KEEP_UNIT_STATIC_GROUP ? !m->grp.at(u.id).cached : !m->seg.at(u.id).cached;
}

int64_t unit_tokens(const keep_memory* m, const UnitRef& u) {
  if (u.kind == KEEP_UNIT_DYNAMIC_SEGMENT) return (int64_t)m->seg.at(u.id).tokens.size();
  int64_t n = 0;
  for (int32_t s : m->grp.at(u.id).segments) n += (int64_t)m->seg.at(s).tokens.size();
  return n;
}

}  // namespace

extern "C" {

keep_status keep_memory_create(int32_t window_t, keep_memory** out) {
  if (!out || window_t < 0) return KEEP_ERR_INVALID_ARG;
  keep_memory* m = new (std::nothrow) keep_memory();
  if (!m) return KEEP_ERR_WORKSPACE;
  m->t = window_t;
  *out = m;
  return KEEP_OK;
}

keep_status keep_memory_destroy(keep_memory* m) {
  delete m;
  return KEEP_OK;
}

const char* keep_memory_last_error(const keep_memory* m) { return m ? m->err.c_str() : "store is NULL"; }

keep_status keep_memory_put(keep_memory* m, int32_t group_id, int32_t segment_id, const int32_t* token_ids,
                            int32_t n_tokens, int32_t* changed) {
  if (!m) return KEEP_ERR_INVALID_ARG;
  if (!token_ids) return mfail(m, KEEP_ERR_INVALID_ARG, "token_ids is NULL");
  if (n_tokens < 1) return mfail(m, KEEP_ERR_INVALID_ARG, "a segment needs at least one token");
  if (group_id < 0 || segment_id < 0) return mfail(m, KEEP_ERR_INVALID_ARG, "ids must be non-negative");
  if (changed) *changed = 1;
  auto it = m->seg.find(segment_id);
  if (it != m->seg.end()) {
    Segment& s = it->second;
    if (s.group != group_id)
      return mfail(m, KEEP_ERR_INVALID_ARG, "segment %d belongs to group %d, not %d", segment_id, s.group, group_id);
    if ((int32_t)s.tokens.size() == n_tokens && std::equal(s.tokens.begin(), s.tokens.end(), token_ids)) {
      if (changed) *changed = 0;
      return KEEP_OK;
    }
    s.tokens.assign(token_ids, token_ids + n_tokens);
    s.last_change = m->now;
    s.cached = false;
    m->grp[group_id].cached = false;
    return KEEP_OK;
  }
  auto gi = m->grp.find(group_id);
  if (gi == m->grp.end()) gi = m->grp.emplace(group_id, Group()).first;
  Group& g = gi->second;
  g.segments.insert(segment_id);
  g.last_member_change = m->now;
  g.cached = false;
  Segment s;
  s.group = group_id;
  s.tokens.assign(token_ids, token_ids + n_tokens);
  s.last_change = m->now;
  s.cached = false;
  m->seg.emplace(segment_id, std::move(s));
  m->units_valid = false;
  return KEEP_OK;
}

keep_status keep_memory_remove(keep_memory* m, int32_t segment_id) {
  if (!m) return KEEP_ERR_INVALID_ARG;
  auto it = m->seg.find(segment_id);
  if (it == m->seg.end()) return mfail(m, KEEP_ERR_INVALID_ARG, "no segment %d", segment_id);
  const int32_t gid = it->second.group;
  m->seg.erase(it);
  Group& g = m->grp[gid];
  g.segments.erase(segment_id);
  g.last_member_change = m->now;
  g.cached = false;
  if (g.segments.empty()) m->grp.erase(gid);
  m->units_valid = false;
  return KEEP_OK;
}

keep_status keep_memory_end_step(keep_memory* m, keep_memory_step_report* report, int32_t* to_dynamic,
                                 int32_t cap_to_dynamic, int32_t* to_static, int32_t cap_to_static) {
  if (!m) return KEEP_ERR_INVALID_ARG;
  int n_td = 0, n_ts = 0, n_sta = 0, n_dyn = 0;
  for (auto& ge : m->grp) {
    Group& g = ge.second;
    int64_t newest = g.last_member_change;
    for (int32_t s : g.segments) newest = std::max(newest, m->seg[s].last_change);
    const int64_t age = m->now - newest;  // closed steps since the newest change
    const int32_t kind = age >= m->t ? KEEP_UNIT_STATIC_GROUP : KEEP_UNIT_DYNAMIC_SEGMENT;
    if (kind != g.kind) {
      // the cache is recomputed the new way: nothing of the old way stays valid
      g.cached = false;
      for (int32_t s : g.segments) m->seg[s].cached = false;
      g.kind = kind;
      m->units_valid = false;
      if (kind == KEEP_UNIT_STATIC_GROUP) {
        if (to_static && n_ts < cap_to_static) to_static[n_ts] = ge.first;
        ++n_ts;
      } else {
        if (to_dynamic && n_td < cap_to_dynamic) to_dynamic[n_td] = ge.first;
        ++n_td;
      }
    }
    (kind == KEEP_UNIT_STATIC_GROUP ? n_sta : n_dyn) += 1;
  }
  if (report) {
    report->step = (int32_t)m->now;
    report->n_static = n_sta;
    report->n_dynamic = n_dyn;
    report->n_to_dynamic = n_td;
    report->n_to_static = n_ts;
    report->dirty_units = 0;
    report->dirty_tokens = 0;
    for (const UnitRef& u : units_of(m)) {
      if (unit_dirty(m, u)) {
        report->dirty_units += 1;
        report->dirty_tokens += unit_tokens(m, u);
      }
    }
  }
  m->now += 1;
  return KEEP_OK;
}

int32_t keep_memory_unit_count(const keep_memory* m) { return m ? (int32_t)units_of(m).size() : 0; }

keep_status keep_memory_unit_info(const keep_memory* m, int32_t unit, keep_memory_unit* out) {
  if (!m) return KEEP_ERR_INVALID_ARG;
  keep_memory* mm = const_cast<keep_memory*>(m);
  if (!out) return mfail(mm, KEEP_ERR_INVALID_ARG, "out is NULL");
  const auto& us = units_of(m);
  if (unit < 0 || unit >= (int32_t)us.size()) return mfail(mm, KEEP_ERR_INVALID_ARG, "unit %d out of range", unit);
  const UnitRef& u = us[unit];
  out->kind = u.kind;
  out->id = u.id;
  out->group = u.group;
  out->n_segments = u.kind == KEEP_UNIT_STATIC_GROUP ? (int32_t)m->grp.at(u.id).segments.size() : 1;
  out->n_tokens = (int32_t)unit_tokens(m, u);
  out->dirty = unit_dirty(m, u) ? 1 : 0;
  return KEEP_OK;
}

keep_status keep_memory_unit_tokens(const keep_memory* m, int32_t unit, int32_t* out, int32_t cap, int32_t* n_tokens) {
  if (!m) return KEEP_ERR_INVALID_ARG;
  keep_memory* mm = const_cast<keep_memory*>(m);
  const auto& us = units_of(m);
  if (unit < 0 || unit >= (int32_t)us.size()) return mfail(mm, KEEP_ERR_INVALID_ARG, "unit %d out of range", unit);
  if (!out || !n_tokens) return mfail(mm, KEEP_ERR_INVALID_ARG, "out / n_tokens is NULL");
  const UnitRef& u = us[unit];
  const int64_t n = unit_tokens(m, u);
  *n_tokens = (int32_t)n;
  if (n > cap) return mfail(mm, KEEP_ERR_WORKSPACE, "unit %d has %lld tokens, capacity %d", unit, (long long)n, cap);
  int32_t* p = out;
  if (u.kind == KEEP_UNIT_DYNAMIC_SEGMENT) {
    const auto& t = m->seg.at(u.id).tokens;
    std::copy(t.begin(), t.end(), p);
  } else {
    for (int32_t s : m->grp.at(u.id).segments) {
      const auto& t = m->seg.at(s).tokens;
      p = std::copy(t.begin(), t.end(), p);
    }
  }
  return KEEP_OK;
}

keep_status keep_memory_mark_computed(keep_memory* m, int32_t unit) {
  if (!m) return KEEP_ERR_INVALID_ARG;
  const auto& us = units_of(m);
  if (unit < 0 || unit >= (int32_t)us.size()) return mfail(m, KEEP_ERR_INVALID_ARG, "unit %d out of range", unit);
  const UnitRef& u = us[unit];
  if (u.kind == KEEP_UNIT_STATIC_GROUP)
    m->grp[u.id].cached = true;
  else
    m->seg[u.id].cached = true;
  return KEEP_OK;
}

}  // extern "C"
