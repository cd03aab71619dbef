// JSON-schema front end (host only): schema text -> grammar text.
#pragma once
#include <string>

#include "automaton.hpp"

namespace xgm {

// Converts a JSON schema into grammar text whose root rule is `root`.
// Supported: type (a name or a list of names: object, array, string, integer,
// number, boolean, null), properties + required (members appear in the order
// of "properties"; without "required" all of them are required; no further
// members), items + minItems / maxItems (up to 64), enum and const of scalar
// values, anyOf / oneOf (both as a union), true and {} (any value),
// annotations (title, description, default, examples, $schema, $id,
// $comment) are ignored.  Keys and string values of enum / const appear in
// their shortest JSON spelling.  Anything that would change the language and
// is not listed (pattern, format, numeric ranges, $ref, ...) is refused.
// Throws Failure(XGM_ERR_PARSE) with a message.
std::string schema_to_grammar(const std::string& schema_json);

}  // namespace xgm
