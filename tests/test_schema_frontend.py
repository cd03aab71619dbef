"""CPU tests of the JSON-schema front end (xgm_schema_to_grammar).

The grammar text it writes is judged by what it accepts: documents generated
from the schema by definition must be sentences, and mutated documents are
sentences exactly when a validator written here from the definition of the
supported keywords says so (Python's json module reads the document; the
validator also checks what the front end documents as its own rules: members
in the order of "properties", numbers of type integer spelled as integers).
Membership is asked of the library's host matcher and of the oracle's Earley
recogniser, which parses the same grammar text with its own parser."""

import json

import numpy as np
import pytest

import oracle
import paper_2411_15100_amd as xgm
import synth_inputs as si

WS = [" ", "\n", "\t", "\r", "  ", ""]


# ----------------------------------------------------------------- schemas
def to_json_schema(node: dict, rng) -> dict:
    """synth_inputs.random_schema's plain dict -> a JSON schema using the supported keywords."""
    t = node["type"]
    if t == "enum":
        vals = list(node["values"])
        if rng.random() < 0.3:
            vals += [int(rng.integers(-5, 100)), None, True]
        return {"enum": vals}
    if t == "array":
        out = {"type": "array", "items": to_json_schema(node["items"], rng)}
        u = rng.random()
        if u < 0.3:
            out["minItems"] = int(rng.integers(0, 3))
        if 0.2 < u < 0.5:
            out["maxItems"] = out.get("minItems", 0) + int(rng.integers(0, 3))
        return out
    if t == "object":
        props = {k: to_json_schema(v, rng) for k, v in node["properties"]}
        out = {"type": "object", "properties": props}
        if rng.random() < 0.7:
            out["required"] = [k for k in props if rng.random() < 0.5]
        if rng.random() < 0.3:
            out["additionalProperties"] = False
        return out
    if t == "number" and rng.random() < 0.3:
        return {"type": ["number", "null"]}
    if t == "string" and rng.random() < 0.2:
        return {"anyOf": [{"type": "string"}, {"type": "boolean"}, {"const": 7}]}
    return {"type": t, "description": "annotations are ignored"}


HANDWRITTEN = {
    "type": "object",
    "title": "awkward names and values",
    "properties": {
        'qu"ote': {"type": "string"},
        "né\\w\nline": {"enum": ["tab\there", "ünï", "", "\u0001"]},
        "anything": True,
        "free": {},
        "loose object": {"type": "object"},
        "loose array": {"type": "array", "maxItems": 2},
        "empty": {"type": "object", "properties": {}},
        "never more": {"type": "array", "items": {"type": "null"}, "maxItems": 0},
        "all optional": {"type": "object", "properties": {"a": {"type": "integer"}, "b": {"type": "boolean"}}, "required": []},
        "one of": {"oneOf": [{"type": "integer"}, {"type": "array", "items": {"type": "integer"}, "minItems": 2}]},
    },
    "required": ['qu"ote', "empty"],
}


# ------------------------------------------------- documents by definition
def gen_value(schema, rng, depth=0):
    """A Python value valid under the schema (numbers as ('int', text) / ('float', text) to fix their spelling)."""
    if schema is True or schema == {}:
        return rng.choice([None, True, ("int", "0"), "free"]) if depth > 2 else {"k": [("float", "-1.5e+3"), "v"], "z": {}}
    if "const" in schema:
        return wrap(schema["const"])
    if "enum" in schema:
        return wrap(schema["enum"][int(rng.integers(0, len(schema["enum"])))])
    for key in ("anyOf", "oneOf"):
        if key in schema:
            return gen_value(schema[key][int(rng.integers(0, len(schema[key])))], rng, depth + 1)
    t = schema.get("type")
    if isinstance(t, list):
        t = t[int(rng.integers(0, len(t)))]
    if t is None:
        t = "object" if "properties" in schema else "array" if "items" in schema else None
    if t == "string":
        pool = ["", "a", "hello world", "q\"uote", "back\\slash", "ünïcode 中", "line\nbreak", "\u0007"]
        return pool[int(rng.integers(0, len(pool)))]
    if t == "integer":
        return ("int", rng.choice(["0", "-0", "7", "-12", "1234567890123"]))
    if t == "number":
        return (rng.choice(["int", "float"]), rng.choice(["0", "-3", "2.50", "1e9", "-0.1E-2", "6.02e+23"]))
    if t == "boolean":
        return bool(rng.integers(0, 2))
    if t == "null":
        return None
    if t == "array":
        lo = schema.get("minItems", 0)
        hi = schema.get("maxItems", lo + 3)
        n = int(rng.integers(lo, hi + 1))
        item = schema.get("items", True)
        return [gen_value(item, rng, depth + 1) for _ in range(n)]
    if t == "object":
        if "properties" not in schema:
            return {"x": ("int", "1"), "y": [None]}
        req = schema.get("required")
        out = {}
        for k, sub in schema["properties"].items():
            if req is None or k in req or rng.random() < 0.5:
                out[k] = gen_value(sub, rng, depth + 1)
        return out
    raise AssertionError(schema)


def wrap(v):
    if isinstance(v, bool) or v is None or isinstance(v, str):
        return v
    if isinstance(v, int):
        return ("int", str(v))
    if isinstance(v, float):
        return ("float", repr(v))
    raise AssertionError(v)


def serialise(v, rng) -> str:
    w = lambda: WS[int(rng.integers(0, len(WS)))]
    if isinstance(v, tuple):
        return v[1]
    if v is None:
        return "null"
    if v is True:
        return "true"
    if v is False:
        return "false"
    if isinstance(v, str):
        return json.dumps(v, ensure_ascii=False)
    if isinstance(v, list):
        return "[" + w() + (w() + "," + w()).join(serialise(x, rng) for x in v) + w() + "]"
    if isinstance(v, dict):
        return "{" + w() + (w() + "," + w()).join(json.dumps(k, ensure_ascii=False) + w() + ":" + w() + serialise(x, rng)
                                                   for k, x in v.items()) + w() + "}"
    raise AssertionError(v)


# --------------------------------------------------- validator by definition
class Pairs(list):
    """A JSON object as read: the (name, value) pairs in document order."""


def read_document(text: str):
    return json.loads(text, object_pairs_hook=Pairs, parse_int=lambda s: ("int", s), parse_float=lambda s: ("float", s),
                      parse_constant=lambda s: (_ for _ in ()).throw(ValueError(s)))


def same_value(doc, const) -> bool:
    if isinstance(const, bool) or const is None or isinstance(const, str):
        return type(doc) is type(const) and doc == const
    return isinstance(doc, tuple) and doc[1] == (str(const) if isinstance(const, int) else repr(const))


def valid(doc, schema) -> bool:
    if schema is True or schema == {}:
        return True
    if "const" in schema:
        return same_value(doc, schema["const"])
    if "enum" in schema:
        return any(same_value(doc, c) for c in schema["enum"])
    for key in ("anyOf", "oneOf"):
        if key in schema:
            return any(valid(doc, s) for s in schema[key])
    t = schema.get("type")
    if isinstance(t, list):
        return any(valid(doc, dict(schema, type=one)) for one in t)
    if t is None:
        t = "object" if "properties" in schema else "array" if "items" in schema else None
    if t is None:
        return True
    if t == "string":
        return isinstance(doc, str)
    if t == "integer":
        return isinstance(doc, tuple) and doc[0] == "int"
    if t == "number":
        return isinstance(doc, tuple)
    if t == "boolean":
        return isinstance(doc, bool)
    if t == "null":
        return doc is None
    if t == "array":
        if not isinstance(doc, list) or isinstance(doc, Pairs):
            return False
        if len(doc) < schema.get("minItems", 0) or len(doc) > schema.get("maxItems", 1 << 30):
            return False
        return all(valid(x, schema.get("items", True)) for x in doc)
    if t == "object":
        if not isinstance(doc, Pairs):
            return False
        if "properties" not in schema:
            return True
        names = list(schema["properties"])
        req = schema.get("required")
        at = 0  # members come in the order of "properties", each at most once, no others
        for k, v in doc:
            while at < len(names) and names[at] != k:
                if req is None or names[at] in req:
                    return False
                at += 1
            if at == len(names) or not valid(v, schema["properties"][k]):
                return False
            at += 1
        return all(req is not None and n not in req for n in names[at:])
    raise AssertionError(schema)


def mutate_value(v, rng):
    """A structural change somewhere in the value (may or may not keep it valid)."""
    if isinstance(v, dict) and v and rng.random() < 0.8:
        keys = list(v)
        u = rng.random()
        if u < 0.2:
            k = keys[int(rng.integers(0, len(keys)))]
            return {a: b for a, b in v.items() if a != k}
        if u < 0.35:
            perm = [keys[int(i)] for i in rng.permutation(len(keys))]
            return {k: v[k] for k in perm}
        if u < 0.45:
            out = dict(v)
            out["extra"] = None
            return out
        k = keys[int(rng.integers(0, len(keys)))]
        return {a: (mutate_value(b, rng) if a == k else b) for a, b in v.items()}
    if isinstance(v, list) and rng.random() < 0.8:
        u = rng.random()
        if v and u < 0.3:
            return v[:-1]
        if u < 0.6:
            return v + [v[0] if v else None]
        if v:
            i = int(rng.integers(0, len(v)))
            return [mutate_value(x, rng) if j == i else x for j, x in enumerate(v)]
    pool = [None, True, ("int", "5"), ("float", "5.0"), "other", [], {}]
    return pool[int(rng.integers(0, len(pool)))]


def accepted_by_library(g, text: bytes) -> bool:
    m = xgm.Matcher(grammar=g)
    return m.try_accept_bytes(text) == 0 and m.can_terminate()


def check_schema(schema: dict, seed: int, n_docs: int):
    text = xgm.schema_to_grammar(json.dumps(schema, ensure_ascii=False))
    g = xgm.Grammar(text, "root")
    og = oracle.Grammar(text, "root")
    rng = np.random.Generator(np.random.PCG64(seed))
    n_valid = n_invalid = 0
    for _ in range(n_docs):
        value = gen_value(schema, rng)
        doc = serialise(value, rng)
        assert valid(read_document(doc), schema), doc          # the generator follows the definition
        raw = doc.encode("utf-8")
        assert accepted_by_library(g, raw), doc
        assert og.recognize(raw) == 2, doc
        # a structural mutation, judged by the validator
        mdoc = serialise(mutate_value(value, rng), rng)
        want = valid(read_document(mdoc), schema)
        assert accepted_by_library(g, mdoc.encode("utf-8")) == want, mdoc
        assert (og.recognize(mdoc.encode("utf-8")) == 2) == want, mdoc
        n_valid += want
        n_invalid += not want
        # a change of one byte: still JSON and valid, or not a sentence
        b = bytearray(raw)
        if b:
            i = int(rng.integers(0, len(b)))
            b[i] = int(rng.choice(list(b' ,:"{}[]0a\\')))
            try:
                want = valid(read_document(bytes(b).decode("utf-8")), schema)
            except (ValueError, UnicodeDecodeError, RecursionError):
                want = False
            if want and b"\\" in bytes(b):
                continue    # an escape the shortest spelling would not use is outside the front end's rules
            assert accepted_by_library(g, bytes(b)) == want, bytes(b)
    return n_valid, n_invalid


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_random_schemas_accept_exactly_the_valid_documents(seed):
    rng = np.random.Generator(np.random.PCG64(1000 + seed))
    schema = to_json_schema(si.random_schema(seed, max_depth=3, string_heavy=bool(seed % 2)), rng)
    n_valid, n_invalid = check_schema(schema, seed, 25)
    assert n_invalid >= 10


def test_handwritten_schema_with_awkward_names_and_loose_parts():
    n_valid, n_invalid = check_schema(HANDWRITTEN, 5, 60)
    assert n_valid >= 3 and n_invalid >= 20


def test_all_required_schemas_give_the_language_of_the_input_generator():
    """For a schema whose members are all required the front end and synth_inputs' own grammar writer
    must describe the same documents."""
    for seed in (0, 4):
        plain = si.random_schema(seed, max_depth=3)

        def convert(node):
            if node["type"] == "enum":
                return {"enum": list(node["values"])}
            if node["type"] == "array":
                return {"type": "array", "items": convert(node["items"])}
            if node["type"] == "object":
                return {"type": "object", "properties": {k: convert(v) for k, v in node["properties"]}}
            return {"type": node["type"]}

        schema = convert(plain)
        ours = xgm.Grammar(xgm.schema_to_grammar(json.dumps(schema)), "root")
        theirs = xgm.Grammar(si.make_schema_grammar(seed, max_depth=3), "root")
        rng = np.random.Generator(np.random.PCG64(seed))
        for _ in range(15):
            value = gen_value(schema, rng)
            for v in (value, mutate_value(value, rng)):
                raw = serialise(v, rng).encode("utf-8")
                assert accepted_by_library(ours, raw) == accepted_by_library(theirs, raw), raw


@pytest.mark.parametrize("bad", [
    '{"type": "string", "pattern": "a+"}', '{"type": "integer", "minimum": 0}', '{"$ref": "#/defs/x"}',
    '{"type": "object", "properties": {"a": {}}, "additionalProperties": true}',
    '{"type": "object", "properties": {"a": {}}, "required": ["b"]}',
    '{"type": "array", "minItems": 3, "maxItems": 2}', '{"type": "array", "maxItems": 65}',
    '{"type": "array", "items": [{"type": "string"}]}', '{"type": "text"}', '{"enum": []}', '{"enum": [[1]]}',
    'false', '[1]', '{"type": "string"', '{"type": "string"} x', '{"a": 1, "a": 2}', '{"type": "str\\ud800ing"}', '',
])
def test_unsupported_and_malformed_schemas_are_refused(bad):
    with pytest.raises(xgm.XgmError) as e:
        xgm.schema_to_grammar(bad)
    assert e.value.status == -2  # XGM_ERR_PARSE
